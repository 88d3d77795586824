// mrp_verify_accept_static: speculative verification (paper Algorithm 3, the accept test) for callers
// that cannot allocate -- code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc.  It is mrp_verify_accept without a context: the same two kernels, with the per-chunk
// argmax partials in a file-scope device array instead of a context's workspace.
#include "../../include/mrp.h"

#include <mutex>

#include "mrp_kernels.h"

namespace mrp {

namespace {

// (max, argmax) partial per (sequence, draft, vocabulary chunk): floats first, then ints
constexpr size_t SCRATCH_ENTRIES = MRP_VERIFY_STATIC_MAX_ENTRIES;
constexpr size_t SCRATCH_BYTES = SCRATCH_ENTRIES * (sizeof(float) + sizeof(int));

// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is a stand-in for the symbol, not a device address: host code
// uses the address hipGetSymbolAddress returned for the current device (scratch_ptr below).
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void *g_scratch_ptr[MAX_DEVICES] = {};

}  // namespace

// Address of the current device's scratch array, resolved once per device; nullptr on failure.
void *verify_static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace mrp

extern "C" {

size_t mrp_verify_accept_static_scratch_bytes(void) { return mrp::SCRATCH_BYTES; }

int mrp_verify_accept_static(void *stream, int B, int L, int V, int K, const float *verify, const int32_t *draft_pos,
                             const int32_t *draft_tok, int draft_stride, uint8_t *match, int32_t *accept_len,
                             int32_t *correction_tok) {
    using namespace mrp;
    if (!verify || !draft_pos || !draft_tok || !match || !accept_len || !correction_tok) return MRP_ERR_NULL;
    if (B < 0 || L < 1 || L > MRP_MAX_BLOCK_LEN || V < 1 || K < 1 || K > MRP_MAX_HEADS || draft_stride < K ||
        (long)B * K > 65535)
        return MRP_ERR_SHAPE;
    const size_t entries = (size_t)B * K * verify_chunks(V);
    if (entries > SCRATCH_ENTRIES) return MRP_ERR_WORKSPACE;   // beyond the fixed scratch array
    if (V % 4 == 0 && (reinterpret_cast<uintptr_t>(verify) & 15u)) return MRP_ERR_ALIGN;
    if (B == 0) return MRP_OK;
    void *p = verify_static_scratch();
    if (!p) return MRP_ERR_HIP;
    float *wm = static_cast<float *>(p);
    int *wi = reinterpret_cast<int *>(static_cast<unsigned char *>(p) + SCRATCH_ENTRIES * sizeof(float));
    // every entry the second kernel reads is written by the first: nothing has to start at zero
    return launch_verify(B, L, V, K, 0, verify, draft_pos, draft_tok, draft_stride, wm, wi, match, accept_len,
                         correction_tok, nullptr, static_cast<hipStream_t>(stream)) == hipSuccess
               ? MRP_OK
               : MRP_ERR_HIP;
}

}  // extern "C"
