// ks_keyswitch_static: the key-switch for callers that may not allocate device memory and have no workspace to
// hand over (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  Its workspace is a
// file-scope device array that every GPU the library runs on holds until the process ends.
//
// In host code the array's name is only a stand-in for the device symbol: each device has its own copy at its
// own address, resolved once per device with hipGetSymbolAddress (from ks_ctx_create, with that device
// current) and kept in g_scratch_ptr.  Host code below uses that pointer, never the array's name.
#include "ks_internal.hpp"

namespace {

// One bootstrapping-level ciphertext (N = 2^16, L = 24, K = 8, dnum = 3: coefficient copy 24 limbs, raised digits 96,
// accumulators 64, converted limbs 48, packed ciphertext limbs of the accumulators 30 = 262 limbs of 512 KiB).
constexpr size_t kStaticScratchBytes = KS_STATIC_WORKSPACE_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

}  // namespace

hipError_t ks::bind_static_scratch(int device) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[device]) return hipSuccess;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
    return hipSuccess;
}

extern "C" size_t ks_static_workspace_bytes(void) { return kStaticScratchBytes; }

extern "C" int ks_keyswitch_static(const ks_ctx* c, const uint64_t* d, uint32_t ell, const uint64_t* evk, uint64_t* out,
                                   uint32_t batch, void* stream) {
    if (!c || c->device < 0 || c->device >= kMaxDevices) return KS_EINVAL;
    void* ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        ws = g_scratch_ptr[c->device];  // bound when the context was created on that device
    }
    if (!ws) return KS_EWORKSPACE;
    if (batch != 0 && ell >= 1 && ell <= c->L) {
        const size_t need = ks_workspace_bytes(c, KS_OP_KEYSWITCH, ell, batch, 0);
        if (need == 0 || need > kStaticScratchBytes) return KS_EWORKSPACE;  // larger than the library-owned scratch
    }
    // every word of the workspace the chain reads has been written earlier in the same call: nothing to clear
    return ks::keyswitch_impl(c, d, ell, evk, out, batch, ws, kStaticScratchBytes, stream, false);
}
