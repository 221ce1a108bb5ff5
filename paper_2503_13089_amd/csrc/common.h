// Internal declarations shared by the translation units of libcluscomp (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace cc {

constexpr uint32_t kMaxK = 1u << 24;

// Device-side bookkeeping at the start of the workspace (one 256-byte slot).
struct WsHeader {
    uint32_t absmax_bits;      // max over all inputs of the fp32 bit pattern of |x|
    uint32_t refine_count;     // length of the refine list written by the last matrix-core assign
    unsigned long long refined_vectors;
    unsigned long long skipped_vectors;
    unsigned long long assign_calls;
    int32_t fixed_point_exp;
    uint32_t reserved;
};

// Carved view of the caller's workspace.
struct Workspace {
    WsHeader* hdr;
    float* cnorm;              // [K]    ||c_k||^2
    long long* sums;           // [K*d]  fixed-point cluster sums
    uint32_t* counts;          // [K]
    double* partials;          // [partial_slots] per-block partial objective
    uint32_t* refine_list;     // [N]    ids of vectors to re-decide in direct form
    float* fast_best;          // [N]    scratch of the matrix-core assign
    uint32_t partial_slots;
    size_t bytes;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Lays the arrays out behind `base` (which may be NULL for a pure size query).
inline Workspace carve(void* base, uint64_t N, uint32_t d, uint32_t K)
{
    Workspace w{};
    char* p = static_cast<char*>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) { char* q = p ? p + off : nullptr; off += align256(bytes); return q; };
    w.hdr = reinterpret_cast<WsHeader*>(take(sizeof(WsHeader)));
    w.cnorm = reinterpret_cast<float*>(take(size_t(K) * 4));
    w.sums = reinterpret_cast<long long*>(take(size_t(K) * d * 8));
    w.counts = reinterpret_cast<uint32_t*>(take(size_t(K) * 4));
    w.partial_slots = uint32_t((N + 255) / 256 + 1);
    w.partials = reinterpret_cast<double*>(take(size_t(w.partial_slots) * 8));
    w.refine_list = reinterpret_cast<uint32_t*>(take(size_t(N) * 4));
    w.fast_best = reinterpret_cast<float*>(take(size_t(N) * 4));
    w.bytes = off;
    return w;
}

// ---- launchers (each enqueues on `s` and returns the launch status) -------------------------------

// Direct-form E-step over all N vectors. partials may be NULL (no objective wanted).
hipError_t launch_assign_direct(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K,
                                uint32_t* idx, double* partials, uint32_t* n_partials_out, hipStream_t s);

// Sums partials[0..n) in index order into *out (fp64).
hipError_t launch_reduce_partials(const double* partials, uint32_t n, double* out, hipStream_t s);

// Header bookkeeping.
hipError_t launch_reset_header(WsHeader* hdr, hipStream_t s);
hipError_t launch_absmax(const float* X, uint64_t n_floats, WsHeader* hdr, hipStream_t s);
hipError_t launch_bump_assign_calls(WsHeader* hdr, hipStream_t s);

// M-step.
hipError_t launch_update(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, const float* prev,
                         uint32_t K, float* out, uint32_t* counts_out, const Workspace& w, hipStream_t s);

// Reconstruction.
hipError_t launch_decode(const float* C, uint32_t K, uint32_t d, const uint32_t* idx, uint64_t N, float* out,
                         hipStream_t s);

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s);

}  // namespace cc
