// Plan-time specialisation of the kernel templates for chains that are not in the built-in catalogue.
//
// The paper generates a kernel per fused subgraph from GIR templates: a graph structure chosen ahead of
// time, parameters filled in per use (section 6, "GIR-Graph generation").  Here the kernel templates of the
// library play that role.  A chain's lowered micro-programs become the template arguments of the same
// kernels the catalogue instantiates at build time (StaticSpec / StaticList), and the HIP run-time compiler
// instantiates them for gfx950 when the plan is made.  Nothing is traced or searched: the "code generator"
// writes one template-id; shapes and immediates stay run-time arguments, so one compiled kernel serves every
// chain with the same structure.  Compiled kernels are kept for the life of the process.
//
// If the run-time compiler or the kernel headers are not available the planner falls back to the
// run-time-interpreted kernels (still on the GPU); nothing else changes.
#include "pf_jit.h"

#include <dlfcn.h>
#include <hip/hiprtc.h>

#include <dirent.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <sstream>
#include <string>
#include <vector>

namespace pf {

namespace {

std::mutex g_mutex;
std::map<std::string, hipFunction_t> g_cache;  // (device, template-id) -> kernel
uint64_t g_compiles = 0;

// the directory that holds the kernel headers: next to the shared library (<package>/lib -> <package>/csrc),
// unless PF_JIT_INCLUDE names another one
std::string include_dir() {
    if (const char* e = getenv("PF_JIT_INCLUDE"))
        if (*e) return e;
    Dl_info info;
    if (dladdr(reinterpret_cast<const void*>(&include_dir), &info) == 0 || !info.dli_fname) return "";
    std::string lib = info.dli_fname;
    const size_t slash = lib.rfind('/');
    if (slash == std::string::npos) return "";
    return lib.substr(0, slash) + "/../csrc";
}

bool file_exists(const std::string& p) {
    FILE* f = fopen(p.c_str(), "rb");
    if (!f) return false;
    fclose(f);
    return true;
}

// ---- kernels kept on disk between processes (opt-in: PF_JIT_CACHE=<directory>) ----------------------------------
// A file holds one code object and the kernel's symbol in it.  Its name is a 128-bit digest of everything the code
// depends on: the generated source, the template-id, the compiler options, the run-time compiler's version and the
// contents of every kernel header.  A file that does not load (truncated, written by something else) is ignored and
// compiled over; files are written under a temporary name and renamed, so a reader never sees half of one.
struct Digest {
    uint64_t a = 1469598103934665603ull, b = 0x9e3779b97f4a7c15ull;
    void add(const void* data, size_t n) {
        const unsigned char* p = static_cast<const unsigned char*>(data);
        for (size_t i = 0; i < n; ++i) {
            a = (a ^ p[i]) * 1099511628211ull;                 // FNV-1a
            b = (b ^ p[i]) * 0xff51afd7ed558ccdull;            // a second, independent mix
            b ^= b >> 29;
        }
    }
    void add(const std::string& t) {
        const uint64_t n = t.size();
        add(&n, sizeof(n));
        add(t.data(), t.size());
    }
};

bool read_file(const std::string& path, std::vector<char>* out) {
    FILE* f = fopen(path.c_str(), "rb");
    if (!f) return false;
    char buf[65536];
    size_t n;
    out->clear();
    while ((n = fread(buf, 1, sizeof(buf), f)) > 0) out->insert(out->end(), buf, buf + n);
    fclose(f);
    return true;
}

// digest of the kernel headers in `inc` (and of the public header they include), computed once per directory
std::string headers_digest(const std::string& inc) {
    static std::map<std::string, std::string> done;  // (under g_mutex)
    auto it = done.find(inc);
    if (it != done.end()) return it->second;
    std::vector<std::string> names;
    if (DIR* d = opendir(inc.c_str())) {
        while (dirent* e = readdir(d)) {
            const std::string n = e->d_name;
            const size_t dot = n.rfind('.');
            const std::string ext = dot == std::string::npos ? "" : n.substr(dot);
            if (ext == ".hpp" || ext == ".h" || ext == ".inc") names.push_back(n);
        }
        closedir(d);
    }
    std::sort(names.begin(), names.end());
    Digest dg;
    std::vector<char> data;
    for (const std::string& n : names) {
        dg.add(n);
        if (read_file(inc + "/" + n, &data)) dg.add(std::string(data.begin(), data.end()));
    }
    if (read_file(inc + "/../../include/pf_chain.h", &data)) dg.add(std::string(data.begin(), data.end()));
    char text[40];
    snprintf(text, sizeof(text), "%016llx%016llx", (unsigned long long)dg.a, (unsigned long long)dg.b);
    return done[inc] = text;
}

uint64_t g_disk_hits = 0;

std::string list_text(const std::vector<uint32_t>& l) {
    std::ostringstream o;
    o << "pf::StaticList<";
    for (size_t i = 0; i < l.size(); ++i) o << (i ? ", " : "") << l[i] << "u";
    o << ">";
    return o.str();
}

std::string spec_text(const JitSpec& s) {
    std::ostringstream o;
    o << "pf::StaticSpec<" << s.nf << ", " << s.nv << ", " << s.nt << ", " << s.core << ", " << s.gamma << ", " << s.beta << ", "
      << list_text(s.pro) << ", " << list_text(s.epi) << ", " << s.flags << ">";
    return o.str();
}

// Compile `source`, which must define the kernel named by the C++ expression `name_expr`, and return it
// loaded on the current device.
hipFunction_t compile(int device, const std::string& source, const std::string& name_expr, std::string* err) {
    const std::string key = std::to_string(device) + "|" + name_expr;
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_cache.find(key);
    if (it != g_cache.end()) return it->second;
    // Only a compile error is remembered (the same source fails the same way every time); missing headers or a module
    // that does not load may be a passing condition, and remembering it would keep this structure on the interpreter
    // for the life of the process.
    auto fail = [&](const std::string& what, bool remember = false) -> hipFunction_t {
        if (err) *err = what;
        if (remember) g_cache[key] = nullptr;
        return nullptr;
    };
    const std::string inc = include_dir();
    if (inc.empty() || !file_exists(inc + "/pf_row_kernels.hpp")) return fail("kernel headers not found (looked in '" + inc + "')");

    // the same code generation options as the build-time kernels
    const std::string inc_opt = "-I" + inc;
    const char* opts[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", inc_opt.c_str(), "-Wno-pass-failed",
                          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};

    auto finish = [&](hipFunction_t fn) {
        const char* lg = getenv("PF_LOG");
        if (lg && atoi(lg) != 0) {  // registers and scratch of the new kernel: what decides how many waves a SIMD holds
            int regs = 0, scratch = 0;
            (void)hipFuncGetAttribute(&regs, HIP_FUNC_ATTRIBUTE_NUM_REGS, fn);
            (void)hipFuncGetAttribute(&scratch, HIP_FUNC_ATTRIBUTE_LOCAL_SIZE_BYTES, fn);
            fprintf(stderr, "[pf_jit] %s: %d registers, %d bytes of scratch per lane\n", name_expr.c_str(), regs, scratch);
        }
        g_cache[key] = fn;  // the module stays loaded until the process ends
        return fn;
    };

    // a kernel kept on disk by an earlier process?
    std::string cache_file;
    if (const char* dir = getenv("PF_JIT_CACHE")) {
        if (*dir) {
            int major = 0, minor = 0;
            (void)hiprtcVersion(&major, &minor);
            Digest dg;
            dg.add(source);
            dg.add(name_expr);
            for (const char* o : opts)
                if (o != inc_opt.c_str()) dg.add(std::string(o));
            dg.add(headers_digest(inc));
            dg.add(std::to_string(major) + "." + std::to_string(minor));
            char name[64];
            snprintf(name, sizeof(name), "/pf_%016llx%016llx.co", (unsigned long long)dg.a, (unsigned long long)dg.b);
            cache_file = std::string(dir) + name;
            std::vector<char> blob;
            if (read_file(cache_file, &blob) && blob.size() > 12 && memcmp(blob.data(), "PFCO", 4) == 0) {
                uint32_t sym_len = 0;
                memcpy(&sym_len, blob.data() + 4, 4);
                if (sym_len > 0 && (size_t)sym_len + 8 < blob.size()) {
                    const std::string sym(blob.data() + 8, blob.data() + 8 + sym_len);
                    hipModule_t mod = nullptr;
                    hipFunction_t fn = nullptr;
                    if (hipModuleLoadData(&mod, blob.data() + 8 + sym_len) == hipSuccess &&
                        hipModuleGetFunction(&fn, mod, sym.c_str()) == hipSuccess) {
                        ++g_disk_hits;
                        return finish(fn);
                    }
                    (void)hipGetLastError();  // a file that does not load is compiled over below
                }
            }
        }
    }

    hiprtcProgram prog = nullptr;
    if (hiprtcCreateProgram(&prog, source.c_str(), "pf_jit.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS)
        return fail("hiprtcCreateProgram failed");
    hiprtcAddNameExpression(prog, name_expr.c_str());
    const hiprtcResult rc = hiprtcCompileProgram(prog, (int)(sizeof(opts) / sizeof(opts[0])), opts);
    if (rc != HIPRTC_SUCCESS) {
        size_t n = 0;
        std::string log;
        if (hiprtcGetProgramLogSize(prog, &n) == HIPRTC_SUCCESS && n > 1) {
            log.resize(n);
            hiprtcGetProgramLog(prog, &log[0]);
        }
        hiprtcDestroyProgram(&prog);
        return fail("run-time compilation failed: " + log.substr(0, 2000), true);
    }
    const char* lowered = nullptr;
    if (hiprtcGetLoweredName(prog, name_expr.c_str(), &lowered) != HIPRTC_SUCCESS || !lowered) {
        hiprtcDestroyProgram(&prog);
        return fail("cannot resolve the compiled kernel's name");
    }
    const std::string symbol = lowered;
    size_t size = 0;
    if (hiprtcGetCodeSize(prog, &size) != HIPRTC_SUCCESS || size == 0) {
        hiprtcDestroyProgram(&prog);
        return fail("empty code object");
    }
    std::vector<char> code(size);
    hiprtcGetCode(prog, code.data());
    hiprtcDestroyProgram(&prog);
    hipModule_t mod = nullptr;
    hipFunction_t fn = nullptr;
    if (hipModuleLoadData(&mod, code.data()) != hipSuccess) return fail("hipModuleLoadData failed");
    if (hipModuleGetFunction(&fn, mod, symbol.c_str()) != hipSuccess) return fail("hipModuleGetFunction failed");
    ++g_compiles;
    if (!cache_file.empty()) {
        // keep it for later processes: written under a name of its own, then renamed into place
        const std::string tmp = cache_file + "." + std::to_string((long)getpid()) + ".tmp";
        if (FILE* f = fopen(tmp.c_str(), "wb")) {
            const uint32_t sym_len = (uint32_t)symbol.size();
            bool ok = fwrite("PFCO", 1, 4, f) == 4 && fwrite(&sym_len, 4, 1, f) == 1 && fwrite(symbol.data(), 1, sym_len, f) == sym_len &&
                      fwrite(code.data(), 1, code.size(), f) == code.size();
            ok = (fclose(f) == 0) && ok;
            if (!ok || rename(tmp.c_str(), cache_file.c_str()) != 0) (void)remove(tmp.c_str());
        }
    }
    return finish(fn);
}

}  // namespace

bool jit_enabled() {
    const char* e = getenv("PF_JIT");
    if (e && *e && atoi(e) == 0) return false;
    const char* ns = getenv("PF_NO_STATIC");
    if (ns && *ns && atoi(ns) != 0) return false;
    return true;
}

uint64_t jit_disk_hits() {
    std::lock_guard<std::mutex> lock(g_mutex);
    return g_disk_hits;
}

uint64_t jit_compile_count() {
    std::lock_guard<std::mutex> lock(g_mutex);
    return g_compiles;
}

hipFunction_t jit_row_kernel(int device, int dtype, int kc, int rpw, bool wave_rows, bool ragged, int max_threads, int log2_lanes,
                             const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    name << "pf::row_kernel<" << dtype << ", " << kc << ", " << rpw << ", " << spec_text(spec) << ", " << max_threads << ", "
         << (wave_rows ? "true" : "false") << ", " << (ragged ? "true" : "false") << ", " << log2_lanes << ">";
    return compile(device, "#include \"pf_row_kernels.hpp\"\n", name.str(), err);
}

// The row kernel with the shape of one launch as constants (a generated type, named by a hash of its contents).
hipFunction_t jit_row_kernel_const(int device, int dtype, int kc, int rpw, bool wave_rows, bool ragged, int max_threads, int log2_lanes,
                                   const JitSpec& spec, const RowShapeConst& sh, std::string* err) {
    std::ostringstream body;
    body << "    static constexpr bool kConst = true;\n"
         << "    static constexpr unsigned n_inner = " << sh.n_inner << "u, mask_si = " << sh.mask_si << "u, core_mask = " << sh.core_mask
         << "u, vec_plain_all = " << sh.vec_plain_all << "u, waves_per_row = " << sh.waves_per_row << "u, rows_per_block = " << sh.rows_per_block
         << "u;\n    static constexpr unsigned long long rows = " << sh.rows << "ull;\n";
    const std::string text = body.str();
    uint64_t h = 1469598103934665603ull;  // FNV-1a
    for (unsigned char c : text) h = (h ^ c) * 1099511628211ull;
    std::ostringstream type, source, name;
    type << "PfRowShape_" << std::hex << h;
    source << "#include \"pf_row_kernels.hpp\"\nstruct " << type.str() << " {\n" << text << "};\n";
    name << "pf::row_kernel<" << dtype << ", " << kc << ", " << rpw << ", " << spec_text(spec) << ", " << max_threads << ", "
         << (wave_rows ? "true" : "false") << ", " << (ragged ? "true" : "false") << ", " << log2_lanes << ", " << type.str() << ">";
    return compile(device, source.str(), name.str(), err);
}

hipFunction_t jit_row_reduce_kernel(int device, int dtype, int k, bool ragged, const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    name << "pf::row_reduce_kernel<" << dtype << ", " << k << ", " << (ragged ? "true" : "false") << ", " << spec_text(spec) << ">";
    return compile(device, "#include \"pf_row_kernels.hpp\"\n", name.str(), err);
}

hipFunction_t jit_row_stream_kernel(int device, int dtype, bool ragged, const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    name << "pf::row_stream_kernel<" << dtype << ", " << (ragged ? "true" : "false") << ", " << spec_text(spec) << ">";
    return compile(device, "#include \"pf_row_stream.hpp\"\n", name.str(), err);
}

hipFunction_t jit_ew_kernel(int device, int dtype, int k, bool ragged, const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    name << "pf::ew_kernel<" << dtype << ", " << k << ", " << spec_text(spec) << ", " << (ragged ? "true" : "false") << ">";
    return compile(device, "#include \"pf_row_kernels.hpp\"\n", name.str(), err);
}

hipFunction_t jit_perm_kernel(int device, int dtype, int variant, int k, bool ragged, const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    const char* rg = ragged ? "true" : "false";
    if (variant == 2) name << "pf::perm_tile_kernel<" << dtype << ", " << spec_text(spec) << ", " << rg << ">";
    else if (variant == 1) name << "pf::perm_lds_rows_kernel<" << dtype << ", " << spec_text(spec) << ">";
    else name << "pf::perm_rows_kernel<" << dtype << ", " << k << ", " << spec_text(spec) << ", " << rg << ">";
    return compile(device, "#include \"pf_perm_kernels.hpp\"\n", name.str(), err);
}

// The row-permutation kernel with this launch's geometry as constants: a generated type in front of the kernel's
// name, named by a hash of its contents (the cache key is the name expression).
hipFunction_t jit_perm_rows_const(int device, int dtype, int k, const JitSpec& spec, const PermGeom& g, const uint32_t* vec_numel,
                                  const uint32_t* vec_period, std::string* err) {
    std::ostringstream body;
    auto list = [&](const char* what, const uint32_t* v, int n) {
        body << "    static constexpr unsigned " << what << "[" << n << "] = {";
        for (int i = 0; i < n; ++i) body << (i ? ", " : "") << v[i] << "u";
        body << "};\n";
    };
    body << "    static constexpr bool kConst = true;\n    static constexpr int rank = " << g.rank << ";\n";
    list("extent", g.extent, PF_DEV_MAX_RANK);
    list("in_stride", g.in_stride, PF_DEV_MAX_RANK);
    list("out_stride", g.out_stride, PF_DEV_MAX_RANK);
    list("vec_numel", vec_numel, PF_DEV_MAX_VEC);
    list("vec_period", vec_period, PF_DEV_MAX_VEC);
    body << "    static constexpr unsigned in_n_inner = " << g.in_n_inner << "u, out_n_inner = " << g.out_n_inner << "u, total_vecs = " << g.total_vecs
         << "u, epi_full_mask = " << g.epi_full_mask << "u, epi_vec_mask = " << g.epi_vec_mask << "u;\n";
    const std::string text = body.str();
    uint64_t h = 1469598103934665603ull;  // FNV-1a
    for (unsigned char c : text) h = (h ^ c) * 1099511628211ull;
    std::ostringstream type, source, name;
    type << "PfPermGeom_" << std::hex << h;
    source << "#include \"pf_perm_kernels.hpp\"\nstruct " << type.str() << " {\n" << text << "};\n";
    name << "pf::perm_rows_kernel<" << dtype << ", " << k << ", " << spec_text(spec) << ", false, " << type.str() << ">";
    return compile(device, source.str(), name.str(), err);
}

hipFunction_t jit_group_kernel(int device, int dtype, int nv, int phase, int general_parts, const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    name << "pf::group_kernel<" << dtype << ", " << nv << ", " << spec_text(spec) << ", " << phase << ", " << general_parts << ">";
    return compile(device, "#include \"pf_group_kernels.hpp\"\n", name.str(), err);
}

// The one-launch group kernel with the geometry of one launch as constants.
hipFunction_t jit_group_kernel_const(int device, int dtype, int nv, int general_parts, const JitSpec& spec, const GroupGeom& g, uint32_t tiles,
                                     uint32_t grid, uint32_t threads, std::string* err) {
    std::ostringstream body;
    body << "    static constexpr bool kConst = true;\n    static constexpr unsigned samples = " << g.samples << "u, hw = " << g.hw << "u, channels = "
         << g.channels << "u, groups = " << g.groups << "u, cv = " << g.cv << "u, vpg = " << g.vpg << "u, log2_vpg = " << g.log2_vpg
         << "u, pos_per_step = " << g.pos_per_step << "u, pos_per_block = " << g.pos_per_block << "u, lanes_per_group = " << g.lanes_per_group
         << "u, blocks_per_sample = " << g.blocks_per_sample << "u, tiles = " << tiles << "u, grid = " << grid << "u, threads = " << threads << "u;\n";
    const std::string text = body.str();
    uint64_t h = 1469598103934665603ull;  // FNV-1a
    for (unsigned char c : text) h = (h ^ c) * 1099511628211ull;
    std::ostringstream type, source, name;
    type << "PfGroupGeom_" << std::hex << h;
    source << "#include \"pf_group_kernels.hpp\"\nstruct " << type.str() << " {\n" << text << "};\n";
    name << "pf::group_kernel<" << dtype << ", " << nv << ", " << spec_text(spec) << ", 0, " << general_parts << ", " << type.str() << ">";
    return compile(device, source.str(), name.str(), err);
}

hipFunction_t jit_stencil_kernel(int device, int dtype, int variant, int ks, bool ragged, const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    const char* rg = ragged ? ", true>" : ", false>";
    if (variant == 2) name << "pf::dwconv_strided_kernel<" << dtype << ", " << spec_text(spec) << ", " << ks << rg;
    else if (variant == 1) name << "pf::dwconv_staged_kernel<" << dtype << ", " << spec_text(spec) << ", " << ks << rg;
    else name << "pf::dwconv3x3_kernel<" << dtype << ", " << spec_text(spec) << rg;
    return compile(device, "#include \"pf_stencil_kernels.hpp\"\n", name.str(), err);
}

hipFunction_t jit_pool_kernel(int device, int dtype, int nv, int op, bool ragged, const JitSpec& spec, std::string* err) {
    std::ostringstream name;
    name << "pf::pool_kernel<" << dtype << ", " << nv << ", " << spec_text(spec) << ", " << op << (ragged ? ", true>" : ", false>");
    return compile(device, "#include \"pf_pool_kernels.hpp\"\n", name.str(), err);
}

int jit_blocks_per_cu(hipFunction_t fn, int block_threads, uint32_t lds_bytes) {
    int n = 0;
    if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn, block_threads, lds_bytes) != hipSuccess) return 0;
    return n;
}

int jit_scratch_bytes(hipFunction_t fn) {
    int n = 0;
    if (hipFuncGetAttribute(&n, HIP_FUNC_ATTRIBUTE_LOCAL_SIZE_BYTES, fn) != hipSuccess) return 0;
    return n;
}

hipError_t jit_launch(hipFunction_t fn, dim3 grid, dim3 block, uint32_t lds_bytes, void** params, hipStream_t st) {
    return hipModuleLaunchKernel(fn, grid.x, grid.y, grid.z, block.x, block.y, block.z, lds_bytes, st, params, nullptr);
}

}  // namespace pf
