"""Host-side bounds check of a generated kernel whose memory indices depend on the lane and on compile-time
constants only (the per-sample uvw kernels): the HIP source is rewritten into a host program in which every
pointer is bounds-checked, and every lane of every wave runs the kernel body on its own.  Cross-lane operations are
stubbed (they move data, never indices), so the data are meaningless; what is checked is that every global and LDS
access of every lane stays inside its array.  Test infrastructure: nothing in the product imports this."""
import os
import re
import subprocess
import tempfile

_PRE = r'''
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <type_traits>
struct Dim { unsigned x; } threadIdx, blockIdx, gridDim;
template <class T> struct FP {
  T* p; long long off, n; const char* name;
  FP() : p(nullptr), off(0), n(0), name("?") {}
  FP(T* p_, long long n_, const char* nm, long long off_ = 0) : p(p_), off(off_), n(n_), name(nm) {}
  template <class U, class = typename std::enable_if<std::is_same<const U, T>::value>::type>
  FP(const FP<U>& o) : p(o.p), off(o.off), n(o.n), name(o.name) {}
  FP operator+(long long d) const { return FP(p, n, name, off + d); }
  T& operator[](long long i) const {
    const long long j = off + i;
    if (j < 0 || j >= n) { std::printf("OUT OF BOUNDS: %s[%lld] (size %lld), lane %u of block %u\n", name, j, n, threadIdx.x & 63, blockIdx.x); std::exit(3); }
    return p[j];
  }
};
template <class T> struct LDS2 {
  std::vector<T> s; long long cols; const char* name;
  LDS2(long long r, long long c, const char* nm) : s(r * c), cols(c), name(nm) {}
  FP<T> operator[](long long r) {
    if (r < 0 || r * cols >= (long long)s.size()) { std::printf("OUT OF BOUNDS: row %lld of %s\n", r, name); std::exit(3); }
    return FP<T>(s.data() + r * cols, cols, name);
  }
};
#define __builtin_amdgcn_readfirstlane(x) (x)
#define __builtin_amdgcn_wave_barrier() ((void)0)
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
'''

_ATTR = r'(?:__attribute__\(\(amdgpu_waves_per_eu\(\d+\)\)\)\s*)?'


def to_host(src):
    """(host C++ text of the kernel as a plain function, kernel name, threads per workgroup)"""
    lines = src.splitlines()
    head = [l for l in lines if l.startswith("typedef") or l.startswith("#define FMA")]
    k0 = next(i for i, l in enumerate(lines) if l.startswith('extern "C" __global__'))
    body = "\n".join(lines[k0:])
    m = re.match(r'extern "C" __global__ void __launch_bounds__\((\d+)\)\s*' + _ATTR + r'(\w+)\(', body)
    wg, name = int(m.group(1)), m.group(2)
    stubs = ("template <int c> static T dpp_(T v) { return v; }\n"
             "static T lane_(T v, int l) { if (l < 0 || l > 63) { std::printf(\"OUT OF BOUNDS: lane index %d\\n\", l); std::exit(3); } return v; }\n"
             "static T wave_sum(T v) { return v; }\n")
    body = re.sub(r'extern "C" __global__ void __launch_bounds__\(\d+\)\s*' + _ATTR, 'void ', body, count=1)
    body = re.sub(r'const T\* __restrict__ (\w+)', r'FP<const T> \1', body)
    body = re.sub(r'\bT\* __restrict__ (\w+)', r'FP<T> \1', body)
    body = re.sub(r'__shared__ (?:__attribute__\(\(aligned\(16\)\)\) )?T (\w+)\[(\d+)\]\[(\d+)\];', r'LDS2<T> \1(\2, \3, "\1");', body)
    body = re.sub(r'const T\* (\w+) =', r'FP<const T> \1 =', body)
    body = re.sub(r'(?<![\w<])T\* (\w+) =', r'FP<T> \1 =', body)
    body = re.sub(r'asm volatile\([^;]*\);', '', body)
    return "\n".join(head) + "\n" + stubs + body, name, wg


def check(src, row_words, B):
    """Runs the kernel for a batch of B rows.  row_words: words per row of every pointer argument, by name.
    Returns (ok, text): text is the program's last line (the first out-of-bounds access if there is one)."""
    code, name, wg = to_host(src)
    sig = re.search(r'void ' + name + r'\(([^)]*)\)', code, re.S).group(1)
    decl, args = [], []
    for p_ in [q.strip() for q in sig.replace("\n", " ").split(",")]:
        nm = p_.split()[-1]
        if nm == "B":
            args.append("B")
            continue
        const = "const " if "const" in p_ else ""
        decl.append(f'  std::vector<T> s_{nm}((size_t)B * {row_words[nm]}, (T)1); FP<{const}T> a_{nm}(s_{nm}.data(), (long long)s_{nm}.size(), "{nm}");')
        args.append(f"a_{nm}")
    main = (f"\nint main() {{\n  const long long B = {B};\n" + "\n".join(decl) + f"\n  const unsigned waves = {wg} / 64;\n"
            "  gridDim.x = (unsigned)((B + waves - 1) / waves);\n  for (blockIdx.x = 0; blockIdx.x < gridDim.x; ++blockIdx.x)\n"
            f"    for (threadIdx.x = 0; threadIdx.x < {wg}; ++threadIdx.x) {name}({', '.join(args)});\n"
            f'  std::printf("in bounds: {name}\\n");\n  return 0;\n}}\n')
    with tempfile.TemporaryDirectory() as d:
        cpp, exe = os.path.join(d, "k.cpp"), os.path.join(d, "k")
        with open(cpp, "w") as f:
            f.write(_PRE + code + main)
        r = subprocess.run(["g++", "-O0", "-std=c++17", "-w", "-o", exe, cpp], capture_output=True, text=True)
        if r.returncode:
            return False, "host build failed: " + r.stderr[:2000]
        r = subprocess.run([exe], capture_output=True, text=True)
        out = (r.stdout.strip().splitlines() or [""])[-1]
        return r.returncode == 0, out
