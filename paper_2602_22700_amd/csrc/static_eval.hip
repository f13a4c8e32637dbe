// imm_mle_eval_static: the multilinear-extension evaluation of imm_mle_eval for callers that cannot
// allocate.  Same kernels, same arithmetic; the working memory (both eq vectors, the column one also cut into bytes for int8 tables, the vector of
// per-row or per-column partial evaluations, the per-split partial vectors) lives in an array that
// is part of the library's device image instead of in buffers a context allocates.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>

#include "../../include/imm.h"
#include "host_field.h"
#include "internal.h"
#include "kernels.h"

// Every device the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for the symbol lookup below.
static __device__ __align__(256) uint64_t scratch[IMM_STATIC_SCRATCH_BYTES / sizeof(uint64_t)];

namespace imm {
namespace {

constexpr uint64_t kWords = IMM_STATIC_SCRATCH_BYTES / sizeof(uint64_t);
constexpr int kMaxDevices = 64;

std::mutex g_mutex;
uint64_t* g_ptr[kMaxDevices] = {};  // device address of `scratch`, per device; null until looked up

// Sections of the array are laid out on 256-byte boundaries.
inline uint64_t round_up(uint64_t words) { return (words + 31) & ~uint64_t(31); }

}  // namespace

int static_scratch_prepare(int device) {
    if (device < 0 || device >= kMaxDevices) {
        set_last_error("static working memory: device index out of range");
        return IMM_E_HIP;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    if (g_ptr[device]) return IMM_OK;
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
        (void)hipGetLastError();
        return fail_hip(e == hipSuccess ? hipErrorInvalidSymbol : e, "hipGetSymbolAddress(static working memory)");
    }
    g_ptr[device] = static_cast<uint64_t*>(p);
    return IMM_OK;
}

}  // namespace imm

extern "C" int imm_mle_eval_static(void* stream, const void* table_dev, imm_dtype dt, uint64_t rows, uint64_t cols,
                                   uint64_t ld, const uint64_t* pt_rows, const uint64_t* pt_cols, uint64_t* out_dev) {
    using namespace imm;
    if (!table_dev || !out_dev) return IMM_E_NULL;
    const uint64_t lim = 1ull << IMM_MAX_ROUNDS;
    if (rows < 1 || cols < 1 || rows > lim || cols > lim || ld < cols) return IMM_E_SHAPE;
    if (dt < IMM_I8 || dt > IMM_F64P) return IMM_E_DTYPE;
    const int tR = hf::ceil_log2(rows), tC = hf::ceil_log2(cols);
    if ((tR && !pt_rows) || (tC && !pt_cols)) return IMM_E_NULL;
    for (int i = 0; i < tR; ++i)
        if (pt_rows[i] >= hf::P) return IMM_E_SHAPE;
    for (int i = 0; i < tC; ++i)
        if (pt_cols[i] >= hf::P) return IMM_E_SHAPE;

    // Layout of the working memory for this shape, and whether it fits.
    const bool along_rows_first = cols >= 256;  // wide table: reduce every row, then one dot product with eq_rows
    const uint64_t len = along_rows_first ? rows : cols;
    const k::Split sp = along_rows_first ? k::plan_over_cols(rows, cols, (int)dt) : k::plan_over_rows(rows, cols);
    const bool direct = sp.nsplit == 1;  // a single split writes the vector itself
    const uint64_t w_eqx = round_up(1ull << tR), w_eqy = round_up(1ull << tC), w_vec = round_up(len);
    const uint64_t w_part = direct ? 0 : round_up((uint64_t)sp.nsplit * len);
    // an int8 table read along its rows takes the column eq vector cut into byte planes as well
    const bool planes = along_rows_first && dt == IMM_I8 && cols % 16 == 0;
    const uint64_t w_planes = planes ? w_eqy : 0;
    const uint64_t need = w_eqx + w_eqy + w_vec + w_part + w_planes;
    if (need > kWords) {
        char msg[192];
        std::snprintf(msg, sizeof(msg),
                      "imm_mle_eval_static: a %llu x %llu table needs %llu bytes of working memory, the static "
                      "buffer holds %llu; use imm_mle_eval",
                      (unsigned long long)rows, (unsigned long long)cols, (unsigned long long)(need * 8),
                      (unsigned long long)(kWords * 8));
        set_last_error(msg);
        return IMM_E_SHAPE;
    }

    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (int rc = static_scratch_prepare(device)) return rc;
    uint64_t* base = g_ptr[device];  // the array's address on this device: what kernels are given, never its name
    uint64_t* eqx = base;
    uint64_t* eqy = eqx + w_eqx;
    uint64_t* vec = eqy + w_eqy;
    uint64_t* part = vec + w_vec;
    uint32_t* eqy_planes = planes ? reinterpret_cast<uint32_t*>(part + w_part) : nullptr;

    hipStream_t s = static_cast<hipStream_t>(stream);
    k::Point pr{}, pc{};
    for (int i = 0; i < tR; ++i) pr.v[i] = pt_rows[i];
    for (int i = 0; i < tC; ++i) pc.v[i] = pt_cols[i];
    // Nothing in the array has to start at zero: the eq vectors, the partial vectors and the vector
    // of partial evaluations are written in full before they are read.
    if ((e = k::eq_build2(s, pr, tR, eqx, pc, tC, eqy, eqy_planes)) != hipSuccess) return fail_hip(e, "eq_build2");
    if (along_rows_first)
        e = k::reduce_over_cols(s, table_dev, (int)dt, rows, cols, ld, eqy, eqy_planes, direct ? vec : part, sp);
    else
        e = k::reduce_over_rows(s, table_dev, (int)dt, rows, cols, ld, eqx, direct ? vec : part, sp);
    if (e != hipSuccess) return fail_hip(e, "partial evaluation");
    if (!direct && (e = k::combine(s, part, sp.nsplit, len, len, vec)) != hipSuccess) return fail_hip(e, "combine");
    if ((e = k::dot(s, vec, along_rows_first ? eqx : eqy, len, out_dev)) != hipSuccess) return fail_hip(e, "dot");
    return IMM_OK;
}
