// Run-time compilation of generated kernels with hipRTC (paper Sec. 4: the generated kernels
// are compiled by the vendor's run-time compiler through a C++ extension), with a code-object
// cache on disk keyed by a hash of the source and the options.
#include <amd_comgr/amd_comgr.h>
#include <dlfcn.h>
#include <hip/hip_runtime_api.h>
#include <hip/hiprtc.h>
#include <sys/stat.h>
#include <unistd.h>

#include <cstdio>
#include <cstring>
#include <fstream>
#include <sstream>
#include <stdexcept>
#include <string>
#include <vector>

#include "plan.hpp"

namespace cgtp {
namespace {

// Packed fp32 instructions are switched off for all generated code: the kernels are written
// for plain v_fma_f32 and all rates quoted for them assume that.
const char* const kOptions[] = {"--offload-arch=gfx950", "-O3",     "-std=c++17",       "-ffp-contract=off",
                                "-Xclang",               "-target-feature", "-Xclang", "-packed-fp32-ops",
                                // float atomics of the unsorted-edge convolution as hardware instructions (device memory
                                // that is coarse-grained, which is what hipMalloc returns), not compare-and-swap loops
                                "-munsafe-fp-atomics"};
constexpr int kNumOptions = sizeof(kOptions) / sizeof(kOptions[0]);
constexpr int kCheckVersion = 3;   // raise when the screening of compiled code changes: older cache entries are then ignored

uint64_t fnv1a(const std::string& s, uint64_t h = 1469598103934665603ull) {
  for (unsigned char c : s) {
    h ^= c;
    h *= 1099511628211ull;
  }
  return h;
}

std::string cache_dir() {
  if (const char* e = std::getenv("CGTP_CACHE_DIR")) return *e ? std::string(e) : std::string();
  Dl_info info;
  if (dladdr((void*)&fnv1a, &info) && info.dli_fname) {
    std::string p(info.dli_fname);
    size_t s = p.find_last_of('/');
    if (s != std::string::npos) return p.substr(0, s) + "/_jit_cache";
  }
  return std::string();
}

bool read_file(const std::string& path, std::vector<char>& out) {
  std::ifstream f(path, std::ios::binary);
  if (!f) return false;
  f.seekg(0, std::ios::end);
  std::streamoff n = f.tellg();
  if (n <= 0) return false;
  out.resize((size_t)n);
  f.seekg(0);
  f.read(out.data(), n);
  return (bool)f;
}

void write_file_atomic(const std::string& path, const std::vector<char>& data) {
  std::string tmp = path + ".tmp" + std::to_string((long)getpid());
  {
    std::ofstream f(tmp, std::ios::binary);
    if (!f) return;
    f.write(data.data(), (std::streamsize)data.size());
    if (!f) {
      std::remove(tmp.c_str());
      return;
    }
  }
  if (std::rename(tmp.c_str(), path.c_str()) != 0) std::remove(tmp.c_str());
}

std::vector<char> compile(const Kernel& k) {
  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, k.source.c_str(), (k.name + ".hip").c_str(), 0, nullptr, nullptr) != HIPRTC_SUCCESS)
    throw std::runtime_error("hiprtcCreateProgram failed for " + k.name);
  hiprtcResult r = hiprtcCompileProgram(prog, kNumOptions, const_cast<const char**>(kOptions));
  if (r != HIPRTC_SUCCESS) {
    size_t n = 0;
    hiprtcGetProgramLogSize(prog, &n);
    std::string log(n, '\0');
    if (n) hiprtcGetProgramLog(prog, &log[0]);
    hiprtcDestroyProgram(&prog);
    throw std::runtime_error("hipRTC failed for " + k.name + ": " + hiprtcGetErrorString(r) + "\n" + log);
  }
  size_t n = 0;
  hiprtcGetCodeSize(prog, &n);
  std::vector<char> code(n);
  hiprtcGetCode(prog, code.data());
  hiprtcDestroyProgram(&prog);
  return code;
}

// Value of an integer entry of the code object's kernel metadata (a MessagePack map inside the ELF note;
// the key is a short string, the value follows it as a MessagePack unsigned integer).  One kernel per
// code object, so the first occurrence of the key is the one.  Returns -1 when absent.
long metadata_int(const std::vector<char>& code, const char* key) {
  const size_t n = std::strlen(key);
  if (n == 0 || n > 31 || code.size() < n + 2) return -1;
  const unsigned char tag = (unsigned char)(0xa0 | n);  // fixstr header
  for (size_t i = 0; i + n + 1 < code.size(); ++i) {
    if ((unsigned char)code[i] != tag || std::memcmp(&code[i + 1], key, n) != 0) continue;
    size_t at = i + 1 + n;
    unsigned char t = (unsigned char)code[at];
    if (t < 0x80) return t;
    size_t w = t == 0xcc ? 1 : t == 0xcd ? 2 : t == 0xce ? 4 : t == 0xcf ? 8 : 0;
    if (!w || at + w >= code.size()) return -1;
    unsigned long long v = 0;
    for (size_t b = 0; b < w; ++b) v = (v << 8) | (unsigned char)code[at + 1 + b];
    return (long)v;
  }
  return -1;
}

// ---- a check of what the compiler produced -------------------------------------------------------------------
// Lanes leave a lane-divergent loop at different times (exec &= ~done; branch back while exec != 0), so the code
// between the loop's exit and the next write to exec runs with an empty execution mask.  Register-allocator spill
// code has been seen to land there (a lane index copied to an accumulation register, resp. stored to private memory):
// the copy does nothing, the reload returns the register's old content, and an address built from it points anywhere.
// Every freshly compiled code object is therefore disassembled (code object manager, one instruction at a time) and
// refused if a vector instruction sits in such a window.
struct DisCtx {
  const char* bytes;
  uint64_t lo, hi;
  std::string text;
};
uint64_t dis_read(uint64_t from, char* to, uint64_t size, void* ud) {
  auto* c = (DisCtx*)ud;
  if (from < c->lo || from >= c->hi) return 0;
  const uint64_t n = std::min<uint64_t>(size, c->hi - from);
  std::memcpy(to, c->bytes + from, n);
  return n;
}
void dis_print(const char* ins, void* ud) { ((DisCtx*)ud)->text = ins; }
void dis_note(uint64_t, void*) {}

bool starts_with(const std::string& s, const char* p) { return s.compare(0, std::strlen(p), p) == 0; }

// the .text section of an ELF64 little-endian code object: [offset, offset + size)
bool text_section(const std::vector<char>& code, uint64_t& lo, uint64_t& hi) {
  if (code.size() < 64 || std::memcmp(code.data(), "\177ELF", 4) != 0 || code[4] != 2) return false;
  auto u16 = [&](size_t at) { uint16_t v; std::memcpy(&v, &code[at], 2); return v; };
  auto u32 = [&](size_t at) { uint32_t v; std::memcpy(&v, &code[at], 4); return v; };
  auto u64 = [&](size_t at) { uint64_t v; std::memcpy(&v, &code[at], 8); return v; };
  const uint64_t shoff = u64(0x28);
  const unsigned shentsize = u16(0x3a), shnum = u16(0x3c), shstrndx = u16(0x3e);
  if (!shoff || shentsize < 64 || shoff + (uint64_t)shnum * shentsize > code.size() || shstrndx >= shnum) return false;
  const uint64_t str = u64(shoff + (uint64_t)shstrndx * shentsize + 0x18);
  for (unsigned i = 0; i < shnum; ++i) {
    const size_t h = shoff + (size_t)i * shentsize;
    const uint64_t name = str + u32(h);
    if (name + 6 > code.size() || std::memcmp(&code[name], ".text", 6) != 0) continue;
    lo = u64(h + 0x18);
    hi = lo + u64(h + 0x20);
    return hi <= code.size() && lo < hi;
  }
  return false;
}

// All instructions of the code object's .text section as text, in address order.
std::vector<std::string> disassemble(const std::vector<char>& code) {
  DisCtx c{code.data(), 0, 0, {}};
  if (!text_section(code, c.lo, c.hi)) throw std::runtime_error("code object: no .text section found");
  amd_comgr_disassembly_info_t info;
  if (amd_comgr_create_disassembly_info("amdgcn-amd-amdhsa--gfx950", dis_read, dis_print, dis_note, &info) != AMD_COMGR_STATUS_SUCCESS)
    throw std::runtime_error("code object manager: cannot create a gfx950 disassembler");
  std::vector<std::string> ins;
  for (uint64_t at = c.lo; at < c.hi;) {
    uint64_t size = 0;
    c.text.clear();
    if (amd_comgr_disassemble_instruction(info, at, &c, &size) != AMD_COMGR_STATUS_SUCCESS || size == 0) {
      c.text = "?";      // padding or data: keep going word by word
      size = 4;
    }
    size_t b = c.text.find_first_not_of(" \t");
    ins.push_back(b == std::string::npos ? std::string() : c.text.substr(b));
    at += size;
  }
  amd_comgr_destroy_disassembly_info(info);
  return ins;
}

// Does the code change the execution mask anywhere (lane-conditional regions, lane-divergent loops)?
bool writes_execution_mask(const std::vector<std::string>& ins) {
  for (const std::string& t : ins) {
    if (t.find("saveexec") != std::string::npos) return true;
    const size_t sp = t.find(' ');
    if (starts_with(t, "s_") && sp != std::string::npos && t.compare(sp + 1, 4, "exec") == 0) return true;
  }
  return false;
}

// Returns the first offending instruction, or an empty string.
std::string vector_instruction_under_empty_mask(const std::vector<std::string>& ins) {
  for (size_t i = 0; i < ins.size(); ++i) {
    if (!starts_with(ins[i], "s_cbranch_execnz")) continue;
    const long off = std::strtol(ins[i].c_str() + std::strlen("s_cbranch_execnz"), nullptr, 0);
    if (off < 32768) continue;                                  // forward branch: not a loop
    bool divergent = false;
    for (size_t j = i >= 3 ? i - 3 : 0; j < i; ++j) divergent |= starts_with(ins[j], "s_andn2_b64 exec, exec");
    if (!divergent) continue;
    for (size_t j = i + 1; j < ins.size(); ++j) {
      const std::string& t = ins[j];
      const size_t sp = t.find(' ');
      const bool writes_exec = starts_with(t, "s_") && sp != std::string::npos && t.compare(sp + 1, 4, "exec") == 0;
      if (writes_exec || starts_with(t, "s_cbranch") || starts_with(t, "s_branch") || starts_with(t, "s_endpgm") || starts_with(t, "s_setpc")) break;
      const bool vector = starts_with(t, "v_") || starts_with(t, "ds_") || starts_with(t, "global_") || starts_with(t, "scratch_") ||
                          starts_with(t, "buffer_") || starts_with(t, "flat_");
      const bool lane_free = starts_with(t, "v_readlane") || starts_with(t, "v_writelane") || starts_with(t, "v_readfirstlane") || starts_with(t, "v_cmp");
      if (vector && !lane_free) return t;
    }
  }
  return std::string();
}

}  // namespace

// For tests: the same check on a code object in a file.  Empty string: nothing found.
std::string jit_check_code_object(const std::string& path) {
  std::vector<char> code;
  if (!read_file(path, code)) throw std::runtime_error("cannot read " + path);
  return vector_instruction_under_empty_mask(disassemble(code));
}

// device >= 0: compile (or fetch from the cache) and load on that device.
// device == -2: compile into the cache only.  device == -1: nothing.
void jit_compile(Kernel& k, int device) {
  if (device == -1 || k.source.empty()) return;
  // the key covers everything that decides the code: source, options, the run-time compiler's version and the
  // version of the checks a code object has to pass before it is stored
  std::string opts;
  for (int i = 0; i < kNumOptions; ++i) opts += std::string(kOptions[i]) + " ";
  int rtc_major = 0, rtc_minor = 0;
  (void)hiprtcVersion(&rtc_major, &rtc_minor);
  opts += "hiprtc " + std::to_string(rtc_major) + "." + std::to_string(rtc_minor) + " checks " + std::to_string(kCheckVersion) + " ";
  char key[40];
  std::snprintf(key, sizeof key, "%016llx", (unsigned long long)fnv1a(k.source, fnv1a(opts)));
  std::string dir = cache_dir();
  std::string path = dir.empty() ? std::string() : dir + "/" + k.name + "_" + key + ".hsaco";
  std::vector<char> code;
  const bool cached = !path.empty() && read_file(path, code);
  if (!cached) code = compile(k);
  // the check runs on cached objects as well (host only, milliseconds): a file written by another build of the
  // library, or damaged on disk, is screened like fresh code
  std::string bad;
  std::vector<std::string> ins;
  try {
    ins = disassemble(code);
  } catch (const std::exception&) {
    if (!cached) throw;
    code = compile(k);   // unreadable cache entry: compile anew
    ins = disassemble(code);
  }
  bad = vector_instruction_under_empty_mask(ins);
  if (!bad.empty())
    throw RefusedCode(k.name + ": the compiler placed a vector instruction (" + bad + ") behind the exit of a lane-divergent loop, "
                             "where the execution mask is empty; the kernel is not used");
  // Register relocation under a partial execution mask.  When a kernel needs more than the 256 architected vector
  // registers (or private memory), the register allocator moves values between registers, accumulation registers and
  // memory; such a move placed inside a lane-conditional region is executed by the active lanes only, and the
  // compiler has been seen to do that to a value that is live in all lanes (an address: the lanes that skipped the
  // region then loaded from address 0, a GPU memory fault).  The uvu kernels are generated without lane-conditional
  // regions for that reason; code that nevertheless has both is not used.
  if (k.screen_divergence && writes_execution_mask(ins) &&
      (metadata_int(code, ".agpr_count") > 0 || metadata_int(code, ".private_segment_fixed_size") > 0))
    throw RefusedCode(k.name + ": the compiled code changes the execution mask and relocates registers (accumulation registers or "
                               "private memory in use); the kernel is not used");
  if (!cached && !path.empty()) {
    mkdir(dir.c_str(), 0755);
    write_file_atomic(path, code);
  }
  long v_ = metadata_int(code, ".vgpr_count");
  if (v_ >= 0) k.vgprs = (int)v_;
  v_ = metadata_int(code, ".agpr_count");
  if (v_ >= 0) k.agprs = (int)v_;
  v_ = metadata_int(code, ".sgpr_count");
  if (v_ >= 0) k.sgprs = (int)v_;
  v_ = metadata_int(code, ".private_segment_fixed_size");
  if (v_ >= 0) k.scratch = (int)v_;
  v_ = metadata_int(code, ".group_segment_fixed_size");
  if (v_ >= 0) k.lds = (int)v_;
  if (device < 0) return;
  hipError_t e = hipModuleLoadData(&k.module, code.data());
  if (e != hipSuccess) throw std::runtime_error("hipModuleLoadData failed for " + k.name + ": " + hipGetErrorString(e));
  e = hipModuleGetFunction(&k.fn, k.module, k.name.c_str());
  if (e != hipSuccess) throw std::runtime_error("hipModuleGetFunction failed for " + k.name + ": " + hipGetErrorString(e));
  int v = 0;
  if (hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_NUM_REGS, k.fn) == hipSuccess) k.vgprs = v;
  if (hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_SHARED_SIZE_BYTES, k.fn) == hipSuccess) k.lds = v;
  if (hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_LOCAL_SIZE_BYTES, k.fn) == hipSuccess) k.scratch = v;
  int nb = 0;
  if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k.fn, k.wg, 0) == hipSuccess) k.blocks_per_cu = nb;
  if (k.blocks_per_cu <= 0) k.blocks_per_cu = 1;
}

void jit_unload(Kernel& k) {
  if (k.module) (void)hipModuleUnload(k.module);
  k.module = nullptr;
  k.fn = nullptr;
}

}  // namespace cgtp
