// sv_op_sample_static: the accept / reject + draw stage for callers that cannot allocate device memory (code
// under graph capture, serving loops that forbid hipMalloc).  Declared in include/specverify_ops.h.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>

#include "../../include/specverify.h"
#include "../../include/specverify_ops.h"
#include "kernels.h"

// Same kernels as sv_op_sample; their scratch (row statistics, per-chain verdicts, the parts of the race) lives
// in a file-scope device array instead of a caller's buffer.  Every GPU the library runs on holds its own copy
// of the array at its own address until the process ends; the address is looked up once per device.
constexpr int kStaticRows = 4096;        // most logits rows B * (1 + N * k) of one call
constexpr int kStaticChains = 4096;      // most chains B * N of one call
constexpr size_t kStaticScratchBytes = (sizeof(float) * 4 * kStaticRows + 255) / 256 * 256 +
                                       3 * ((sizeof(int32_t) * kStaticChains + 255) / 256 * 256) +
                                       (sizeof(float) * 4 * sv::kDrawParts * kStaticRows + 255) / 256 * 256;
// (No `used` attribute here: with it the compiler keeps the array's internal linkage in the device code object,
// where the runtime then cannot find it by name; referenced from host code alone it is emitted as a global symbol.)
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once looked up
static std::mutex g_scratch_mutex;

// Device address of the static scratch array on the current GPU (nullptr on error).  The array's name is a
// host-side handle, not an address a kernel can use: only the pointer returned here is ever handed to one.
static void* static_scratch_ptr() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

extern "C" int sv_op_sample_static(const float* logits, const int32_t* drafts, const float* draft_probs,
                                   const float* uniforms, const int32_t* draft_lens, int B, int N, int k, int V,
                                   int verify_mode, int sample_mode, float temperature, int32_t* accepted_len,
                                   int32_t* out_tokens, int32_t* best_chain, void* stream) {
    if (B <= 0 || N <= 0 || k < 0) return SV_EINVAL;
    if ((int64_t)B * (1 + (int64_t)N * k) > kStaticRows || (int64_t)B * N > kStaticChains) return SV_EINVAL;   // beyond the static array
    if (sv_op_sample_scratch_bytes(B, N, k) > kStaticScratchBytes) return SV_EINVAL;
    void* ptr = static_scratch_ptr();
    if (!ptr) return SV_EHIP;
    // Nothing in the scratch has to start at zero: every field a kernel of this call reads was written by an
    // earlier kernel of the same call (part statistics -> row statistics -> verdicts -> race parts -> tokens).
    return sv_op_sample(logits, drafts, draft_probs, uniforms, draft_lens, B, N, k, V, verify_mode, sample_mode, temperature,
                        ptr, accepted_len, out_tokens, best_chain, stream);
}
