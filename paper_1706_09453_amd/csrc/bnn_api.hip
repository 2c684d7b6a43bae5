// C ABI of the gfx950 binary-network forward pass: argument checks, kernel selection, launches.
// See include/bnn.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstring>

#include "../../include/bnn.h"
#include "mfma32_kernels.hpp"
#include "mfma_i8_kernels.hpp"
#include "realx_mfma_kernels.hpp"
#include "realw_kernels.hpp"
#include "realw_split_kernels.hpp"
#include "mfma_kernels.hpp"
#include "pack_kernels.hpp"
#include "realx_fused_kernel.hpp"
#include "realx_slab_kernels.hpp"
#include "realx_i8_gemm_kernels.hpp"
#include "softmax_kernels.hpp"
#include "train_kernels.hpp"
#include "valu_kernels.hpp"

#define BNN_EXPORT extern "C" __attribute__((visibility("default")))

// Hand-over area of the cooperative log-Softmax epilogue (BNN_OPT_COOPERATIVE): a fixed array in the library's device
// image, kCoopSlots launches' worth, handed out round-robin, so that the tail of one launch and the head of the next
// on another stream do not share a slot.  In host code the array's name is only a handle for hipGetSymbolAddress.
constexpr int kCoopSlots = 4;
constexpr int kCoopMaxTiles = 1024;                                         // workgroups of one cooperative launch, at most
constexpr size_t kCoopFlagBytes = (size_t)kCoopMaxTiles * 8;
constexpr size_t kCoopPairBytes = (size_t)kCoopMaxTiles * 256 * 8;         // 256 rows per tile, 8 bytes per (max, sum) pair
constexpr size_t kCoopSlotBytes = kCoopFlagBytes + kCoopPairBytes;
static __device__ __align__(256) unsigned char coop_area[256 + kCoopSlots * kCoopSlotBytes];   // [0, 4): timeouts

namespace {

using namespace bnn;

// Tuning knobs (bnn_set_option).  Plain atomics: set from the host thread that benchmarks.
std::atomic<int> g_default_arm{BNN_ARM_MFMA};
std::atomic<int> g_realx_tm{0};
std::atomic<int> g_binx_valu_tm{16};
std::atomic<int> g_mfma_wm{4};
std::atomic<int> g_realx_sign_mfma{1};
std::atomic<int> g_fused_softmax{0};
std::atomic<int> g_mfma_shape{0};
std::atomic<int> g_mfma32_wm{0};
std::atomic<int> g_mfma32_pipeline{0};
std::atomic<int> g_realx_f32_mfma{0};
std::atomic<int> g_mfma32_xcd_order{0};
std::atomic<int> g_stream_max_frames{64};
std::atomic<int> g_realx_i8_lsm{1};
std::atomic<int> g_realw_split_lsm{1};
std::atomic<int> g_realw_valu_lds{1};
std::atomic<int> g_cooperative{0};
std::atomic<int> g_coop_spin{1 << 20};
std::atomic<int> g_mfma32_splitk{0};

std::atomic<unsigned long long> g_coop_launches{0};
constexpr int kCoopMaxDevices = 64;
std::atomic<void*> g_coop_ptr[kCoopMaxDevices];
std::atomic<int> g_coop_capacity[kCoopMaxDevices][2];   // resident workgroups of the cooperative kernel, [0/1 input]

// Device address of coop_area on the current device (looked up once per device); *dev_out = that device.
unsigned char* coop_base(int* dev_out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kCoopMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    *dev_out = dev;
    void* p = g_coop_ptr[dev].load(std::memory_order_acquire);
    if (p) return static_cast<unsigned char*>(p);
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(coop_area)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_coop_ptr[dev].store(p, std::memory_order_release);
    return static_cast<unsigned char*>(p);
}

inline bool word_bits_ok(int wb) { return wb == 32 || wb == 64; }
inline int64_t words_per_row(int64_t K, int wb) { return (K + wb - 1) / wb; }
// Row length in 32-bit words (a 64-bit word is two little-endian 32-bit words).
inline int64_t row_w32(int64_t K, int wb) { return words_per_row(K, wb) * (wb / 32); }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline bool overlap(const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return na && nb && a0 < b0 + nb && b0 < a0 + na;
}
inline int launch_status() { return hipGetLastError() == hipSuccess ? BNN_OK : BNN_EDEVICE; }

constexpr int64_t kMaxDim = (int64_t)1 << 30;
constexpr int64_t kMaxN = (int64_t)1 << 22;   // outputs of a layer: the second grid dimension (65535) counts tiles of 128 or 256 of them

size_t out_bytes(int64_t M, int64_t N, int act, int wb) {
    if (act == BNN_ACT_SIGN) return (size_t)M * (size_t)row_w32(N, wb) * 4;
    return (size_t)M * (size_t)N * 4;
}

int check_layer_args(const void* X, const void* Wp, int64_t M, int64_t K, int64_t N, int act, int wb, const void* Y,
                     bool binx, bool realw = false) {
    if (!word_bits_ok(wb) || M < 0 || K <= 0 || N <= 0 || M > kMaxDim || K > kMaxDim || N > kMaxN) return BNN_ESHAPE;
    if (binx && K >= ((int64_t)1 << 24)) return BNN_ESHAPE;
    if (act < BNN_ACT_RAW_I32 || act > BNN_ACT_SIGMOID) return BNN_EINVAL;
    if (!binx && act == BNN_ACT_RAW_I32) return BNN_EINVAL;
    if (M == 0) return BNN_OK;
    if (!X || !Wp || !Y) return BNN_EINVAL;
    if (!aligned(Wp, realw ? 4 : wb / 8)) return BNN_EALIGN;
    if (!aligned(X, binx ? wb / 8 : 4)) return BNN_EALIGN;
    if (!aligned(Y, act == BNN_ACT_SIGN ? wb / 8 : 4)) return BNN_EALIGN;
    const size_t xb = binx ? (size_t)M * row_w32(K, wb) * 4 : (size_t)M * K * 4;
    const size_t wbytes = realw ? (size_t)N * K * 4 : (size_t)N * row_w32(K, wb) * 4;
    const size_t yb = out_bytes(M, N, act, wb);
    if (overlap(X, xb, Y, yb) || overlap(Wp, wbytes, Y, yb)) return BNN_EINVAL;
    return BNN_OK;
}

// ---------------------------------------------------------------- launches (arguments already checked)

template <int TM, bool BCAST>
void launch_realx_tm_b(const float* X, const uint32_t* Wp, const float* scale, const float* bias, int M, int K, int N,
                       int w32, int act, void* Y, int yw32, hipStream_t st) {
    const dim3 grid((M + TM - 1) / TM, (N + 255) / 256), block(256);
    switch (act) {
        case BNN_ACT_SIGN:
            realx_valu_kernel<TM, ACT_SIGN, BCAST><<<grid, block, 0, st>>>(X, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_HARDTANH:
            realx_valu_kernel<TM, ACT_HARDTANH, BCAST><<<grid, block, 0, st>>>(X, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_SIGMOID:
            realx_valu_kernel<TM, ACT_SIGMOID, BCAST><<<grid, block, 0, st>>>(X, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        default:
            realx_valu_kernel<TM, ACT_LINEAR, BCAST><<<grid, block, 0, st>>>(X, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
    }
}

// the row-broadcast variant reads 16 bytes of a frame per lane: rows 16-byte aligned
template <int TM>
void launch_realx_tm(const float* X, const uint32_t* Wp, const float* scale, const float* bias, int M, int K, int N,
                     int w32, int act, void* Y, int yw32, hipStream_t st) {
    if ((K & 3) == 0 && aligned(X, 16)) launch_realx_tm_b<TM, true>(X, Wp, scale, bias, M, K, N, w32, act, Y, yw32, st);
    else launch_realx_tm_b<TM, false>(X, Wp, scale, bias, M, K, N, w32, act, Y, yw32, st);
}

// The fp32 matrix-core kernel runs one workgroup per CU (measured: 1.06 ms with two against 0.54 ms on 432 workgroups);
// the kernel's own occupancy attribute says so.
template <int ACT, bool VEC, bool WREAL>
void launch_f32_mfma(dim3 grid, dim3 block, hipStream_t st, const float* X, const void* W, const float* scale,
                     const float* bias, int M, int K, int N, int w32, float* Y) {
    realx_f32_mfma_kernel<ACT, VEC, WREAL><<<grid, block, 0, st>>>(X, W, scale, bias, M, K, N, w32, Y);
}

void launch_log_softmax(float* Z, int M, int N, hipStream_t st) {
    const dim3 grid(M < 65536 ? M : 65536), block(256);
    const bool al = aligned(Z, 16);
    if (al && N <= 1024) log_softmax_rows_reg_kernel<4><<<grid, block, 0, st>>>(Z, M, N);
    else if (al && N <= 2048) log_softmax_rows_reg_kernel<8><<<grid, block, 0, st>>>(Z, M, N);
    else if (al && N <= 4096) log_softmax_rows_reg_kernel<16><<<grid, block, 0, st>>>(Z, M, N);
    else if (al && N <= 8192) log_softmax_rows_reg_kernel<32><<<grid, block, 0, st>>>(Z, M, N);
    else log_softmax_rows_kernel<<<grid, block, 0, st>>>(Z, M, N);
}

int run_realx(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M, int64_t K, int64_t N,
              int act, int wb, void* Y, hipStream_t st) {
    if (M == 0) return BNN_OK;
    const int w32 = (int)row_w32(K, wb), yw32 = (int)row_w32(N, wb);
    const uint32_t* W = static_cast<const uint32_t*>(Wp);
    const int f32_mfma = g_realx_f32_mfma.load();
    if (act != BNN_ACT_SIGN && M >= 128 && (f32_mfma == 1 || (f32_mfma == 0 && act == BNN_ACT_LOGSOFTMAX))) {
        // fp32 outputs of a large batch on the matrix cores (fp32 MFMA, weights as +-1.0f).  By default only where
        // nothing but the log-Softmax follows; Sign bits never come here
        const dim3 grid((unsigned)((M + 255) / 256), (unsigned)((N + 127) / 128)), block(256);
        const bool vec = (K % 16 == 0) && aligned(X, 16);
        float* Yf = static_cast<float*>(Y);
        if (act == BNN_ACT_HARDTANH) {
            if (vec) launch_f32_mfma<ACT_HARDTANH, true, false>(grid, block, st, X, W, scale, bias, (int)M, (int)K, (int)N, w32, Yf);
            else launch_f32_mfma<ACT_HARDTANH, false, false>(grid, block, st, X, W, scale, bias, (int)M, (int)K, (int)N, w32, Yf);
        } else if (act == BNN_ACT_SIGMOID) {
            if (vec) launch_f32_mfma<ACT_SIGMOID, true, false>(grid, block, st, X, W, scale, bias, (int)M, (int)K, (int)N, w32, Yf);
            else launch_f32_mfma<ACT_SIGMOID, false, false>(grid, block, st, X, W, scale, bias, (int)M, (int)K, (int)N, w32, Yf);
        } else {
            if (vec) launch_f32_mfma<ACT_LINEAR, true, false>(grid, block, st, X, W, scale, bias, (int)M, (int)K, (int)N, w32, Yf);
            else launch_f32_mfma<ACT_LINEAR, false, false>(grid, block, st, X, W, scale, bias, (int)M, (int)K, (int)N, w32, Yf);
        }
        if (act == BNN_ACT_LOGSOFTMAX) launch_log_softmax(Yf, (int)M, (int)N, st);
        return launch_status();
    }
    // batches of a few frames (streaming): 1 or 2 frames per workgroup spread the layer over the chip
    int tm = M <= g_stream_max_frames.load() ? (M <= 16 ? 1 : 2) : g_realx_tm.load();
    if (tm == 0 && ((M + 15) / 16) * ((N + 1023) / 1024) < 256) {
        // too few frames for 16 x 1024 tiles to give every CU a workgroup: the row-broadcast kernel with the most
        // frames per workgroup (fewest sign-building instructions per fma) that still gives 256 workgroups
        tm = 16;
        while (tm > 2 && ((M + tm - 1) / tm) * ((N + 255) / 256) < 256) tm >>= 1;
    }
    if (tm == 0 && (K & 3) == 0 && aligned(X, 16)) {
        // large batch, aligned rows: frames through LDS, every fma on three VGPRs
        constexpr int TM = 16, TNN = 4;
        const int Mi = (int)M, Ki = (int)K, Ni = (int)N;
        const dim3 grid((unsigned)((M + TM - 1) / TM), (unsigned)((N + 256 * TNN - 1) / (256 * TNN))), block(256);
        switch (act) {
            case BNN_ACT_SIGN: realx_valu_lds_kernel<TM, TNN, ACT_SIGN><<<grid, block, 0, st>>>(X, W, scale, bias, Mi, Ki, Ni, w32, Y, yw32); break;
            case BNN_ACT_HARDTANH: realx_valu_lds_kernel<TM, TNN, ACT_HARDTANH><<<grid, block, 0, st>>>(X, W, scale, bias, Mi, Ki, Ni, w32, Y, yw32); break;
            case BNN_ACT_SIGMOID: realx_valu_lds_kernel<TM, TNN, ACT_SIGMOID><<<grid, block, 0, st>>>(X, W, scale, bias, Mi, Ki, Ni, w32, Y, yw32); break;
            default: realx_valu_lds_kernel<TM, TNN, ACT_LINEAR><<<grid, block, 0, st>>>(X, W, scale, bias, Mi, Ki, Ni, w32, Y, yw32); break;
        }
        if (act == BNN_ACT_LOGSOFTMAX) launch_log_softmax(static_cast<float*>(Y), Mi, Ni, st);
        return launch_status();
    }
    switch (tm) {
        case 1: launch_realx_tm<1>(X, W, scale, bias, (int)M, (int)K, (int)N, w32, act, Y, yw32, st); break;
        case 2: launch_realx_tm<2>(X, W, scale, bias, (int)M, (int)K, (int)N, w32, act, Y, yw32, st); break;
        case 4: launch_realx_tm<4>(X, W, scale, bias, (int)M, (int)K, (int)N, w32, act, Y, yw32, st); break;
        case 8: launch_realx_tm<8>(X, W, scale, bias, (int)M, (int)K, (int)N, w32, act, Y, yw32, st); break;
        case 32: launch_realx_tm<32>(X, W, scale, bias, (int)M, (int)K, (int)N, w32, act, Y, yw32, st); break;
        default: launch_realx_tm<16>(X, W, scale, bias, (int)M, (int)K, (int)N, w32, act, Y, yw32, st); break;
    }
    if (act == BNN_ACT_LOGSOFTMAX) launch_log_softmax(static_cast<float*>(Y), (int)M, (int)N, st);
    return launch_status();
}

template <int TM, int ACT, int KC>
void launch_realw_valu_tm(const float* X, const float* W, const float* bias, int M, int K, int N, void* Y, int yw32,
                          hipStream_t st) {
    const dim3 grid((M + TM - 1) / TM, (N + 255) / 256), block(256);
    if ((K & 3) == 0 && aligned(X, 16) && aligned(W, 16)) {
        constexpr unsigned lds = realw_lds_bytes(KC);
        if (lds > 64 * 1024) {   // LDS above 64 KiB has to be allowed once per kernel and device
            static std::atomic<uint64_t> allowed{0};
            int dev = 0;
            (void)hipGetDevice(&dev);
            const uint64_t bit = 1ull << (dev & 63);
            if (!(allowed.load() & bit)) {
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&realw_valu_kernel<TM, ACT, KC>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                allowed.fetch_or(bit);
            }
        }
        realw_valu_kernel<TM, ACT, KC><<<grid, block, lds, st>>>(X, W, bias, M, K, N, Y, yw32);
    } else {
        realw_valu_simple_kernel<TM, ACT><<<grid, block, 0, st>>>(X, W, bias, M, K, N, Y, yw32);
    }
}

// batches of a few frames (streaming): 2 frames per workgroup, so that the layer is spread over ceil(M / 2) x N / 256
// workgroups (up to 16 frames with chunks of 64 k: fewer memory round trips, but 136 KiB of LDS, one workgroup per CU;
// measured at 64 frames: 134 us with chunks of 16 k, 151 us with 64); otherwise 16 frames per workgroup
template <int ACT>
void launch_realw_valu(const float* X, const float* W, const float* bias, int M, int K, int N, void* Y, int yw32,
                       hipStream_t st) {
    if (M <= g_stream_max_frames.load() && M <= 16) launch_realw_valu_tm<2, ACT, 64>(X, W, bias, M, K, N, Y, yw32, st);
    else if (M <= g_stream_max_frames.load()) launch_realw_valu_tm<2, ACT, 16>(X, W, bias, M, K, N, Y, yw32, st);
    else if (M >= 2048 && getenv("BNN_REALW_TM32")) launch_realw_valu_tm<32, ACT, 16>(X, W, bias, M, K, N, Y, yw32, st);
    else launch_realw_valu_tm<16, ACT, 16>(X, W, bias, M, K, N, Y, yw32, st);
}

template <int ACT>
void launch_realw_mfma(const float* X, const float* W, const float* bias, int M, int K, int N, float* Y, hipStream_t st) {
    const dim3 grid((unsigned)((M + 255) / 256), (unsigned)((N + 127) / 128)), block(256);
    if ((K % 16 == 0) && aligned(X, 16) && aligned(W, 16))
        launch_f32_mfma<ACT, true, true>(grid, block, st, X, W, nullptr, bias, M, K, N, 0, Y);
    else
        launch_f32_mfma<ACT, false, true>(grid, block, st, X, W, nullptr, bias, M, K, N, 0, Y);
}

// A layer with real-valued weights.  The matrix-core rule is the one of run_realx.
int run_realw(const float* X, const float* W, const float* bias, int64_t M, int64_t K, int64_t N, int act, int wb,
              void* Y, hipStream_t st) {
    if (M == 0) return BNN_OK;
    const int yw32 = (int)row_w32(N, wb);
    const int f32_mfma = g_realx_f32_mfma.load();
    if (act == BNN_ACT_LOGSOFTMAX && f32_mfma != 2 && M <= 64 && M <= g_stream_max_frames.load() && (K & 3) == 0 &&
        aligned(X, 16) && aligned(W, 16)) {
        // a few frames in front of the log-Softmax: K split over the lanes, so that N / 4 waves pull the weights
        float* Yf = static_cast<float*>(Y);
        const unsigned nb = (unsigned)((N + 15) / 16);
        if (M <= 4) realw_gemv_kernel<4><<<dim3(nb, (unsigned)((M + 3) / 4)), 256, 0, st>>>(X, W, bias, (int)M, (int)K, (int)N, Yf);
        else realw_gemv_kernel<8><<<dim3(nb, (unsigned)((M + 7) / 8)), 256, 0, st>>>(X, W, bias, (int)M, (int)K, (int)N, Yf);
    } else if (act != BNN_ACT_SIGN && M >= 128 && (f32_mfma == 1 || (f32_mfma == 0 && act == BNN_ACT_LOGSOFTMAX))) {
        float* Yf = static_cast<float*>(Y);
        if (act == BNN_ACT_HARDTANH) launch_realw_mfma<ACT_HARDTANH>(X, W, bias, (int)M, (int)K, (int)N, Yf, st);
        else if (act == BNN_ACT_SIGMOID) launch_realw_mfma<ACT_SIGMOID>(X, W, bias, (int)M, (int)K, (int)N, Yf, st);
        else launch_realw_mfma<ACT_LINEAR>(X, W, bias, (int)M, (int)K, (int)N, Yf, st);
    } else {
        switch (act) {
            case BNN_ACT_SIGN: launch_realw_valu<ACT_SIGN>(X, W, bias, (int)M, (int)K, (int)N, Y, yw32, st); break;
            case BNN_ACT_HARDTANH: launch_realw_valu<ACT_HARDTANH>(X, W, bias, (int)M, (int)K, (int)N, Y, yw32, st); break;
            case BNN_ACT_SIGMOID: launch_realw_valu<ACT_SIGMOID>(X, W, bias, (int)M, (int)K, (int)N, Y, yw32, st); break;
            default: launch_realw_valu<ACT_LINEAR>(X, W, bias, (int)M, (int)K, (int)N, Y, yw32, st); break;
        }
    }
    if (act == BNN_ACT_LOGSOFTMAX) launch_log_softmax(static_cast<float*>(Y), (int)M, (int)N, st);
    return launch_status();
}

int run_unpack(const void* Xp, int64_t M, int64_t K, int wb, int zero_one, float* X, hipStream_t st) {
    if (M == 0) return BNN_OK;
    const int64_t total = M * K;
    const int64_t blocks = (total + 255) / 256;
    bits_to_real_kernel<<<(unsigned)(blocks < 65536 ? blocks : 65536), 256, 0, st>>>(static_cast<const uint32_t*>(Xp), M, (int)K,
                                                                                     (int)row_w32(K, wb), zero_one, X);
    return launch_status();
}

template <int TM, bool VEC4, bool X01 = false>
void launch_binx_valu_tm(const uint32_t* Xp, const uint32_t* Wp, const float* scale, const float* bias, int M, int K,
                         int N, int w32, int act, void* Y, int yw32, hipStream_t st) {
    const dim3 grid((M + TM - 1) / TM, (N + 255) / 256), block(256);
    switch (act) {
        case BNN_ACT_RAW_I32:
            binx_valu_kernel<TM, ACT_RAW_I32, VEC4, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_SIGN:
            binx_valu_kernel<TM, ACT_SIGN, VEC4, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_HARDTANH:
            binx_valu_kernel<TM, ACT_HARDTANH, VEC4, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_SIGMOID:
            binx_valu_kernel<TM, ACT_SIGMOID, VEC4, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        default:
            binx_valu_kernel<TM, ACT_LINEAR, VEC4, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
    }
}

template <int WM, bool AL>
void launch_binx_mfma_wm(const uint32_t* Xp, const uint32_t* Wp, const float* scale, const float* bias, int M, int K,
                         int N, int w32, int act, void* Y, int yw32, hipStream_t st) {
    constexpr int WN = 4;
    const dim3 grid((M + 32 * WM - 1) / (32 * WM), (N + 32 * WN - 1) / (32 * WN)), block(256);
    switch (act) {
        case BNN_ACT_RAW_I32:
            binx_mfma_kernel<WM, WN, ACT_RAW_I32, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_SIGN:
            binx_mfma_kernel<WM, WN, ACT_SIGN, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_HARDTANH:
            binx_mfma_kernel<WM, WN, ACT_HARDTANH, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_SIGMOID:
            binx_mfma_kernel<WM, WN, ACT_SIGMOID, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        default:
            binx_mfma_kernel<WM, WN, ACT_LINEAR, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
    }
}

template <int WM, bool AL, bool PP = false, bool X01 = false>
void launch_binx_mfma32(const uint32_t* Xp, const uint32_t* Wp, const float* scale, const float* bias, int M, int K, int N,
                        int w32, int act, void* Y, int yw32, hipStream_t st, const CoopLsm& coop = CoopLsm{}) {
    constexpr int WN = 2;
    // XCD-aware tile order pays when the default order thrashes the per-XCD L2s (a frames operand of more than
    // 8 x 4 MiB) or scatters a large packed output with long rows over many passes; it costs 5-15 % on mid-size
    // problems (measured on MI355X), so it is chosen by size unless forced.
    const int xsel = g_mfma32_xcd_order.load();
    const int xo = xsel == 1 || (xsel == 0 && ((size_t)M * w32 * 4 > ((size_t)32 << 20) ||
                                              (N >= 4096 && (size_t)M * N / 8 >= ((size_t)32 << 20))));
    const unsigned int ab = (unsigned int)((size_t)M * w32 * 4), bb = (unsigned int)((size_t)N * w32 * 4);   // used by the PP variants only
    const dim3 grid((M + 64 * WM - 1) / (64 * WM), (N + 64 * WN - 1) / (64 * WN)), block(256);
    switch (act) {
        case ACT_LSM_COOP:
            if constexpr (WM == 4 && AL && PP)
                binx_mfma32_kernel<WM, WN, ACT_LSM_COOP, AL, PP, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32, ab, bb, xo, coop);
            break;
        case ACT_DOT_I16:
            binx_mfma32_kernel<WM, WN, ACT_DOT_I16, AL, PP, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32, ab, bb, xo, coop);
            break;
        case BNN_ACT_RAW_I32:
            binx_mfma32_kernel<WM, WN, ACT_RAW_I32, AL, PP, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32, ab, bb, xo, coop);
            break;
        case BNN_ACT_SIGN:
            binx_mfma32_kernel<WM, WN, ACT_SIGN, AL, PP, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32, ab, bb, xo, coop);
            break;
        case BNN_ACT_HARDTANH:
            binx_mfma32_kernel<WM, WN, ACT_HARDTANH, AL, PP, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32, ab, bb, xo, coop);
            break;
        case BNN_ACT_SIGMOID:
            binx_mfma32_kernel<WM, WN, ACT_SIGMOID, AL, PP, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32, ab, bb, xo, coop);
            break;
        default:
            binx_mfma32_kernel<WM, WN, ACT_LINEAR, AL, PP, X01><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32, ab, bb, xo, coop);
            break;
    }
}

template <bool AL>
void launch_binx_mfma_i8(const uint32_t* Xp, const uint32_t* Wp, const float* scale, const float* bias, int M, int K, int N,
                         int w32, int act, void* Y, int yw32, hipStream_t st) {
    const dim3 grid((M + 127) / 128, (N + 127) / 128), block(256);
    switch (act) {
        case BNN_ACT_RAW_I32:
            binx_mfma_i8_kernel<ACT_RAW_I32, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_SIGN:
            binx_mfma_i8_kernel<ACT_SIGN, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_HARDTANH:
            binx_mfma_i8_kernel<ACT_HARDTANH, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        case BNN_ACT_SIGMOID:
            binx_mfma_i8_kernel<ACT_SIGMOID, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
        default:
            binx_mfma_i8_kernel<ACT_LINEAR, AL><<<grid, block, 0, st>>>(Xp, Wp, scale, bias, M, K, N, w32, Y, yw32);
            break;
    }
}

int run_binx(const void* Xp, const void* Wp, const float* scale, const float* bias, int64_t M, int64_t K, int64_t N,
             int act, int wb, void* Y, int arm, hipStream_t st, bool x01 = false) {
    if (M == 0) return BNN_OK;
    const bool stream = arm == BNN_ARM_AUTO && M <= g_stream_max_frames.load();
    if (arm == BNN_ARM_AUTO) arm = g_default_arm.load();
    if (x01) arm = BNN_ARM_MFMA;   // large batches: the 0/1 reading of the input bits exists on the 32x32x64 kernel only
    const int w32 = (int)row_w32(K, wb), yw32 = (int)row_w32(N, wb);
    const uint32_t* A = static_cast<const uint32_t*>(Xp);
    const uint32_t* B = static_cast<const uint32_t*>(Wp);
    const bool rows16 = (w32 % 4 == 0) && aligned(Xp, 16) && aligned(Wp, 16);
    const int Mi = (int)M, Ki = (int)K, Ni = (int)N;
    if (stream) {
        // Batches of a few frames (streaming): the matrix-core tiles would be nearly empty and a workgroup would
        // still walk all of K for its 64 or 128 rows.  The vector-ALU kernel with 1 or 2 frames per workgroup spreads
        // the layer over ceil(M / TM) x N / 256 workgroups, each of which is done after one pass over its weight rows.
        auto go = [&](auto tmc, auto vec, auto z1) {
            launch_binx_valu_tm<decltype(tmc)::value, decltype(vec)::value, decltype(z1)::value>(A, B, scale, bias, Mi, Ki, Ni, w32,
                                                                                                act, Y, yw32, st);
        };
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        const bool one = M <= 16;
        if (rows16) {
            if (x01) { if (one) go(I1{}, std::true_type{}, std::true_type{}); else go(I2{}, std::true_type{}, std::true_type{}); }
            else { if (one) go(I1{}, std::true_type{}, std::false_type{}); else go(I2{}, std::true_type{}, std::false_type{}); }
        } else {
            if (x01) { if (one) go(I1{}, std::false_type{}, std::true_type{}); else go(I2{}, std::false_type{}, std::true_type{}); }
            else { if (one) go(I1{}, std::false_type{}, std::false_type{}); else go(I2{}, std::false_type{}, std::false_type{}); }
        }
    } else if (arm == BNN_ARM_VALU_XOR) {
        const int tm = g_binx_valu_tm.load();
        if (rows16) {
            if (tm == 1) launch_binx_valu_tm<1, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else if (tm == 2) launch_binx_valu_tm<2, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else if (tm == 4) launch_binx_valu_tm<4, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else if (tm == 8) launch_binx_valu_tm<8, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else if (tm == 32) launch_binx_valu_tm<32, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else launch_binx_valu_tm<16, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        } else {
            if (tm == 8) launch_binx_valu_tm<8, false>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else if (tm == 32) launch_binx_valu_tm<32, false>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else launch_binx_valu_tm<16, false>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        }
    } else if (arm == BNN_ARM_MFMA_I8) {
        if (rows16 && K % 512 == 0) launch_binx_mfma_i8<true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        else launch_binx_mfma_i8<false>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
    } else if (!x01 && act == BNN_ACT_LOGSOFTMAX && g_fused_softmax.load() && rows16 &&
               ((K % 512 == 0 && N <= 16 * 8 * 16) || (K % 256 == 0 && N <= 16 * 8 * 32)) &&
               (size_t)(M + 16) * w32 * 4 < 0x7fffffffu && (size_t)(N + 512) * w32 * 4 < 0x7fffffffu) {
        // output layer: product, affine step and log-Softmax fused, one workgroup per 16 frames
        const int nf = (int)((N + 127) / 128);
        const dim3 grid((Mi + 15) / 16), block(512);
        float* Yf = static_cast<float*>(Y);
        const unsigned int ab = (unsigned int)((size_t)M * w32 * 4), bb = (unsigned int)((size_t)N * w32 * 4);
        if (K % 512 == 0 && nf <= 8)
            binx_mfma_logsoftmax_kernel<8, 4><<<grid, block, 0, st>>>(A, B, scale, bias, Mi, Ki, Ni, w32, Yf, ab, bb);
        else if (K % 512 == 0 && nf <= 16)
            binx_mfma_logsoftmax_kernel<16, 4><<<grid, block, 0, st>>>(A, B, scale, bias, Mi, Ki, Ni, w32, Yf, ab, bb);
        else if (nf <= 28)
            binx_mfma_logsoftmax_kernel<28, 2><<<grid, block, 0, st>>>(A, B, scale, bias, Mi, Ki, Ni, w32, Yf, ab, bb);
        else
            binx_mfma_logsoftmax_kernel<32, 2><<<grid, block, 0, st>>>(A, B, scale, bias, Mi, Ki, Ni, w32, Yf, ab, bb);
        return launch_status();
    } else if (x01 || g_mfma_shape.load() == 32 || (g_mfma_shape.load() == 0 && M >= 1024)) {
        // large batch: 32x32x64 MFMA, 128 x 64 (or 64 x 64) wave tiles
        const bool al = rows16 && (K % 512 == 0);
        // Output layer: the product goes to memory as int16 (half the bytes of fp32 pre-activations), and the row
        // kernel forms fma(scale, dot, bias) itself before the log-Softmax.
        const bool i16 = act == BNN_ACT_LOGSOFTMAX && K < 32768 && N % 4 == 0 && N <= 8192 && aligned(Y, 16) &&
                         (!scale || aligned(scale, 16)) && (!bias || aligned(bias, 16));
        if (i16) act = ACT_DOT_I16;
        const int64_t tiles_n4 = (N + 127) / 128, tiles4 = ((M + 255) / 256) * tiles_n4;
        // 128-row wave tiles expand fewer operand words per MAC; 64-row ones give twice the workgroups, which
        // matters more while the 128-row grid leaves CUs without a workgroup (measured on MI355X: 64-row tiles win
        // up to 2048 frames x 2048 outputs, 128-row tiles from 4096 x 2048 on)
        const int64_t blocks4 = ((M + 255) / 256) * ((N + 127) / 128);
        const int wm32 = g_mfma32_wm.load();
        const bool wm2 = wm32 == 2 || (wm32 == 0 && blocks4 < 200);
        // fetch pinned ahead of the products: faster on every shape measured; buffer addressing needs operands below 2 GiB
        const bool pinned = g_mfma32_pipeline.load() != 2 && (size_t)M * w32 * 4 < 0x7fffffffu && (size_t)N * w32 * 4 < 0x7fffffffu;
        // Cooperative log-Softmax (opt-in): the product kernel finishes the rows itself.  Its workgroups wait for each
        // other, so all of them have to be resident at once.
        CoopLsm coop{};
        if ((act == BNN_ACT_LOGSOFTMAX || act == ACT_DOT_I16) && g_cooperative.load() && al && pinned && !wm2 && tiles_n4 <= 64 &&
            tiles4 <= kCoopMaxTiles) {
            int dev = -1;
            unsigned char* base = coop_base(&dev);
            int cap = base ? g_coop_capacity[dev][x01 ? 1 : 0].load() : 0;
            if (base && cap == 0) {
                int per_cu = 0, cus = 0;
                const hipError_t e1 = x01 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, binx_mfma32_kernel<4, 2, ACT_LSM_COOP, true, true, true>, 256, 0)
                                          : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, binx_mfma32_kernel<4, 2, ACT_LSM_COOP, true, true, false>, 256, 0);
                const hipError_t e2 = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
                if (e1 != hipSuccess || e2 != hipSuccess) (void)hipGetLastError();
                cap = (e1 == hipSuccess && e2 == hipSuccess && per_cu > 0 && cus > 0) ? per_cu * cus : -1;
                g_coop_capacity[dev][x01 ? 1 : 0].store(cap);
            }
            if (base && tiles4 <= cap) {
                const unsigned long long launch = ++g_coop_launches;
                unsigned char* slot = base + 256 + (size_t)(launch % kCoopSlots) * kCoopSlotBytes;
                coop.flags = reinterpret_cast<unsigned long long*>(slot);
                coop.partials = reinterpret_cast<float2*>(slot + kCoopFlagBytes);
                coop.stamp = launch;
                coop.timeouts = reinterpret_cast<unsigned int*>(base);
                coop.spin_limit = g_coop_spin.load();
                act = ACT_LSM_COOP;
            }
        }
        if (x01) {
            if (!al) launch_binx_mfma32<2, false, false, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else if (!pinned) launch_binx_mfma32<2, true, false, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);   // operands of 2 GiB or more: pointer addressing
            else if (wm2) launch_binx_mfma32<2, true, true, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else launch_binx_mfma32<4, true, true, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st, coop);
        } else if (!al) {
            // ragged rows: bounds-checked word loads, 64-row wave tiles only
            launch_binx_mfma32<2, false>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        } else if (wm2) {
            if (pinned) launch_binx_mfma32<2, true, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else launch_binx_mfma32<2, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        } else if (act == BNN_ACT_SIGN && pinned && K % 1024 == 0 && g_mfma32_splitk.load() == 1) {
            // two waves per SIMD from a grid of one workgroup per CU, by splitting K inside the workgroup (comparison
            // arm: measured slower at Config 3's size, see the option)
            const int xsel = g_mfma32_xcd_order.load();
            const int xo = xsel == 1 || (xsel == 0 && ((size_t)M * w32 * 4 > ((size_t)32 << 20) ||
                                                      (N >= 4096 && (size_t)M * N / 8 >= ((size_t)32 << 20))));
            const dim3 grid((Mi + 255) / 256, (Ni + 127) / 128), block(512);
            binx_mfma32_kernel<4, 2, ACT_SIGN, true, true, false, true><<<grid, block, 0, st>>>(
                A, B, scale, bias, Mi, Ki, Ni, w32, Y, yw32, (unsigned int)((size_t)M * w32 * 4), (unsigned int)((size_t)N * w32 * 4), xo, CoopLsm{});
        } else {
            if (pinned) launch_binx_mfma32<4, true, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st, coop);
            else launch_binx_mfma32<4, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        }
    } else {
        const bool al = rows16 && (K % 512 == 0);
        const int wm = g_mfma_wm.load();
        if (al) {
            if (wm == 2) launch_binx_mfma_wm<2, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else launch_binx_mfma_wm<4, true>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        } else {
            if (wm == 2) launch_binx_mfma_wm<2, false>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
            else launch_binx_mfma_wm<4, false>(A, B, scale, bias, Mi, Ki, Ni, w32, act, Y, yw32, st);
        }
    }
    if (act == BNN_ACT_LOGSOFTMAX) launch_log_softmax(static_cast<float*>(Y), Mi, Ni, st);
    if (act == ACT_DOT_I16) {
        constexpr int ROWS = 1;   // two rows per workgroup (shared scale/bias loads) measured slower
        const int nblk = (Mi + ROWS - 1) / ROWS;
        const dim3 grid(nblk < 65536 ? nblk : 65536), block(256);
        float* Z = static_cast<float*>(Y);
        if (Ni <= 1024) log_softmax_rows_i16_kernel<4, ROWS><<<grid, block, 0, st>>>(Z, scale, bias, Mi, Ni);
        else if (Ni <= 2048) log_softmax_rows_i16_kernel<8, ROWS><<<grid, block, 0, st>>>(Z, scale, bias, Mi, Ni);
        else if (Ni <= 4096) log_softmax_rows_i16_kernel<16, ROWS><<<grid, block, 0, st>>>(Z, scale, bias, Mi, Ni);
        else log_softmax_rows_i16_kernel<32, ROWS><<<grid, block, 0, st>>>(Z, scale, bias, Mi, Ni);
    }
    return launch_status();
}

int run_pack(const float* X, int64_t rows, int64_t K, int wb, void* out, hipStream_t st) {
    if (rows == 0) return BNN_OK;
    const int64_t chunks = (K + 63) / 64;
    const int64_t tasks = rows * chunks;
    int64_t blocks = (tasks + 3) / 4;
    if (blocks > 65536 * 4) blocks = 65536 * 4;
    pack_sign_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(X, rows, K, row_w32(K, wb),
                                                                    static_cast<uint32_t*>(out));
    return launch_status();
}

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The matrix-core path of a real-input Sign layer (first layer of a binary-activation network) applies when
// K is small enough for its integer arithmetic; it needs no scratch in global memory.
bool realx_sign_mfma_applies(const bnn_layer_desc& d) {
    return !d.x_is_binary && d.act == BNN_ACT_SIGN && d.K <= kRealxMfmaMaxK;
}

int run_realx_sign_mfma(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M, int64_t K,
                        int64_t N, int wb, void* Y, hipStream_t st) {
    const int Mi = (int)M, Ki = (int)K, Ni = (int)N;
    const int w32 = (int)row_w32(K, wb), yw32 = (int)row_w32(N, wb);
    const int kpad = (Ki + 63) / 64 * 64;
    int nb = (Ni + kRealxChunk - 1) / kRealxChunk * kRealxChunk;
    if (nb > kRealxMaxNB) nb = kRealxMaxNB;
    const size_t lds = realx_dynamic_lds(Ki, kpad, w32, nb);
    const dim3 grid((Mi + kRealxBM - 1) / kRealxBM, (Ni + nb - 1) / nb), block(kRealxThreads);
    // More than 64 KB of LDS per workgroup has to be requested explicitly (gfx950 has 160 KB per CU).
    static std::atomic<size_t> granted_vec{48 * 1024}, granted_scalar{48 * 1024};
    const bool vec16 = aligned(Wp, 16);   // chunks start at multiples of 512 rows: 16-byte aligned whenever the matrix is
    std::atomic<size_t>& granted = vec16 ? granted_vec : granted_scalar;
    if (lds > granted.load()) {
        const void* fn = vec16 ? reinterpret_cast<const void*>(realx_sign_fused_kernel<true>)
                               : reinterpret_cast<const void*>(realx_sign_fused_kernel<false>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return BNN_EDEVICE;
        }
        granted.store(lds);
    }
    if (vec16)
        realx_sign_fused_kernel<true><<<grid, block, lds, st>>>(X, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki, kpad,
                                                               Ni, nb, w32, static_cast<uint32_t*>(Y), yw32);
    else
        realx_sign_fused_kernel<false><<<grid, block, lds, st>>>(X, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki, kpad,
                                                                Ni, nb, w32, static_cast<uint32_t*>(Y), yw32);
    return launch_status();
}

// The same filter for any real-input Sign layer (any position in the network, K up to kSlabMaxK): the frames are
// quantised into digit planes in the caller's workspace first, then K streams through LDS in slabs.
bool realx_sign_slab_applies(const bnn_layer_desc& d) {
    return !d.x_is_binary && !d.w_is_real && d.act == BNN_ACT_SIGN && d.K <= kSlabMaxK;
}
size_t realx_sign_slab_bytes(int64_t M, int64_t K) {
    const size_t kpad = (size_t)(K + 63) / 64 * 64;
    return (kDigits * (size_t)M * kpad + 255) / 256 * 256 + ((size_t)M * sizeof(RowMeta) + 255) / 256 * 256;
}
int run_realx_sign_slab(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M, int64_t K,
                        int64_t N, int wb, void* Y, void* scratch_mem, hipStream_t st) {
    const int Mi = (int)M, Ki = (int)K, Ni = (int)N;
    const int w32 = (int)row_w32(K, wb), yw32 = (int)row_w32(N, wb);
    const int kpad = (Ki + 63) / 64 * 64;
    int8_t* planes = static_cast<int8_t*>(scratch_mem);
    RowMeta* meta = reinterpret_cast<RowMeta*>(planes + (kDigits * (size_t)M * kpad + 255) / 256 * 256);
    if (Ki % 4 == 0 && Ki <= 2048 && aligned(X, 16))
        realx_quantize_kernel<true><<<dim3((Mi + 3) / 4), dim3(256), 0, st>>>(X, Mi, Ki, kpad, slab_quant_bits(Ki), planes, meta);
    else
        realx_quantize_kernel<false><<<dim3((Mi + 3) / 4), dim3(256), 0, st>>>(X, Mi, Ki, kpad, slab_quant_bits(Ki), planes, meta);
    const size_t lds = slab_dynamic_lds();
    const bool vec16 = aligned(Wp, 16) && (w32 % 4 == 0);
    static std::atomic<int> granted[2] = {{0}, {0}};   // more than 64 KB of LDS per workgroup has to be requested explicitly
    if (!granted[vec16].load()) {
        const void* fn = vec16 ? reinterpret_cast<const void*>(realx_sign_slab_kernel<true>)
                               : reinterpret_cast<const void*>(realx_sign_slab_kernel<false>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return BNN_EDEVICE;
        }
        granted[vec16].store(1);
    }
    const dim3 grid((Mi + kRealxBM - 1) / kRealxBM, (Ni + kSlabNB - 1) / kSlabNB), block(kSlabThreads);
    if (vec16)
        realx_sign_slab_kernel<true><<<grid, block, lds, st>>>(X, planes, meta, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki,
                                                              kpad, Ni, w32, static_cast<uint32_t*>(Y), yw32);
    else
        realx_sign_slab_kernel<false><<<grid, block, lds, st>>>(X, planes, meta, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki,
                                                               kpad, Ni, w32, static_cast<uint32_t*>(Y), yw32);
    return launch_status();
}

// Output layer with real inputs and binary weights on the int8 matrix cores (four digit planes), inside bnn_forward
// (the planes live in the workspace): product kernel, then the log-Softmax row kernel.
bool realx_i8_lsm_applies(const bnn_layer_desc& d, int64_t M) {
    return !d.x_is_binary && !d.w_is_real && d.act == BNN_ACT_LOGSOFTMAX && d.K <= kSlabMaxK && M >= 128;
}
size_t realx_i8_lsm_bytes(int64_t M, int64_t K) {
    const size_t kpad = (size_t)(K + 63) / 64 * 64;
    return (kDigits4 * (size_t)M * kpad + 255) / 256 * 256 + ((size_t)M * sizeof(RowMeta4) + 255) / 256 * 256;
}
int run_realx_i8_lsm(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M, int64_t K, int64_t N,
                     int wb, float* Y, void* scratch_mem, hipStream_t st) {
    const int Mi = (int)M, Ki = (int)K, Ni = (int)N;
    const int w32 = (int)row_w32(K, wb);
    const int kpad = (Ki + 63) / 64 * 64;
    int8_t* planes = static_cast<int8_t*>(scratch_mem);
    RowMeta4* meta = reinterpret_cast<RowMeta4*>(planes + (kDigits4 * (size_t)M * kpad + 255) / 256 * 256);
    realx_quantize4_kernel<<<dim3((Mi + 3) / 4), dim3(256), 0, st>>>(X, Mi, Ki, kpad, planes, meta);
    const size_t lds = slab4_dynamic_lds();
    const bool vec16 = aligned(Wp, 16) && (w32 % 4 == 0);
    static std::atomic<int> granted[2] = {{0}, {0}};
    if (!granted[vec16].load()) {
        const void* fn = vec16 ? reinterpret_cast<const void*>(realx_i8_linear_kernel<true>)
                               : reinterpret_cast<const void*>(realx_i8_linear_kernel<false>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return BNN_EDEVICE;
        }
        granted[vec16].store(1);
    }
    const dim3 grid((Mi + kRealxBM - 1) / kRealxBM, (Ni + kSlabNB - 1) / kSlabNB), block(kSlabThreads);
    if (vec16)
        realx_i8_linear_kernel<true><<<grid, block, lds, st>>>(X, planes, meta, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki,
                                                              kpad, Ni, w32, Y);
    else
        realx_i8_linear_kernel<false><<<grid, block, lds, st>>>(X, planes, meta, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki,
                                                               kpad, Ni, w32, Y);
    launch_log_softmax(Y, Mi, Ni, st);
    return launch_status();
}

// Softmax layer with real weights on the bf16 matrix cores (three bf16 pieces per operand, six piece products), inside
// bnn_forward (the planes of both operands live in the workspace): two split passes, the product kernel, then the
// log-Softmax row kernel.  `scratch_mem` is 256-byte aligned.
bool realw_split_lsm_applies(const bnn_layer_desc& d, int64_t M) {
    return d.w_is_real && d.act == BNN_ACT_LOGSOFTMAX && M >= 128;
}
size_t realw_split_planes_bytes(int64_t rows, int64_t K) {
    return (kSplitPieces * (size_t)rows * (size_t)split_kpad((int)K) * 2 + 255) / 256 * 256;
}
size_t realw_split_lsm_bytes(int64_t M, int64_t K, int64_t N) {
    return realw_split_planes_bytes(M, K) + realw_split_planes_bytes(N, K);
}
void launch_split(const float* A, int64_t rows, int K, int kpad, uint16_t* planes, hipStream_t st) {
    const int64_t blocks = (rows * (kpad / 8) + 255) / 256;
    const unsigned grid = (unsigned)(blocks < 16384 ? blocks : 16384);
    if ((K & 3) == 0 && aligned(A, 16)) split_bf16x3_kernel<true><<<grid, 256, 0, st>>>(A, rows, K, kpad, planes);
    else split_bf16x3_kernel<false><<<grid, 256, 0, st>>>(A, rows, K, kpad, planes);
}
int run_realw_split_lsm(const float* X, const float* W, const float* bias, int64_t M, int64_t K, int64_t N, float* Y,
                        void* scratch_mem, hipStream_t st) {
    const int Mi = (int)M, Ki = (int)K, Ni = (int)N;
    const int kpad = split_kpad(Ki);
    uint16_t* xs = static_cast<uint16_t*>(scratch_mem);
    uint16_t* ws = reinterpret_cast<uint16_t*>(static_cast<char*>(scratch_mem) + realw_split_planes_bytes(M, K));
    launch_split(X, M, Ki, kpad, xs, st);
    launch_split(W, N, Ki, kpad, ws, st);
    const unsigned lds = split_dynamic_lds();
    const int eight = g_realw_split_lsm.load() == 2;   // 4 x 2 waves of 64 x 64 (two per SIMD) instead of 2 x 2 waves of 128 x 64
    static std::atomic<int> granted[2] = {{0}, {0}};   // more than 64 KB of LDS per workgroup has to be requested explicitly
    if (!granted[eight].load()) {
        const void* fn = eight ? reinterpret_cast<const void*>(realw_bf16x3_kernel<ACT_LINEAR, 8>)
                               : reinterpret_cast<const void*>(realw_bf16x3_kernel<ACT_LINEAR, 4>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return BNN_EDEVICE;
        }
        granted[eight].store(1);
    }
    const dim3 grid((unsigned)((Mi + kSplitTileM - 1) / kSplitTileM), (unsigned)((Ni + kSplitTileN - 1) / kSplitTileN));
    if (eight) realw_bf16x3_kernel<ACT_LINEAR, 8><<<grid, 512, lds, st>>>(xs, ws, bias, Mi, kpad, Ni, Y);
    else realw_bf16x3_kernel<ACT_LINEAR, 4><<<grid, 256, lds, st>>>(xs, ws, bias, Mi, kpad, Ni, Y);
    launch_log_softmax(Y, Mi, Ni, st);
    return launch_status();
}

// Layers with real weights whose outputs are not log-Softmax inputs, 512 frames or more, inside bnn_forward: the
// ascending-k chains of realw_valu_kernel on fmas with three register operands (realw_valu_lds_kernel), from a
// transposed copy of the weights in the workspace (kpad x N fp32, 256-byte aligned; K padded to 64).
bool realw_valu_lds_applies(const bnn_layer_desc& d, int64_t M) {
    // (the limits keep the grids of both kernels and the 32-bit byte offset inside a row of the copy in range)
    return d.w_is_real && d.act != BNN_ACT_LOGSOFTMAX && M >= 512 && (d.K & 3) == 0 && d.K <= 65536 && d.N <= (1 << 22);
}
size_t realw_valu_lds_bytes(int64_t K, int64_t N) {
    return round_up((size_t)realw_lds_kpad((int)K) * (size_t)N * 4, 256);
}
template <int ACT>
void launch_realw_valu_lds(const float* X, const float* Wt, const float* bias, int M, int K, int kpad, int N, void* Y, int yw32,
                           hipStream_t st) {
    const dim3 grid((unsigned)((M + kRealwLdsFrames - 1) / kRealwLdsFrames), (unsigned)((N + 255) / 256));
    realw_valu_lds_kernel<ACT><<<grid, 256, 0, st>>>(X, Wt, bias, M, K, kpad, N, Y, yw32);
}
int run_realw_valu_lds(const float* X, const float* W, const float* bias, int64_t M, int64_t K, int64_t N, int act, int wb, void* Y,
                       void* scratch_mem, hipStream_t st) {
    const int Mi = (int)M, Ki = (int)K, Ni = (int)N, kpad = realw_lds_kpad(Ki);
    const int yw32 = (int)row_w32(N, wb);
    float* Wt = static_cast<float*>(scratch_mem);
    weights_transposed_kernel<<<dim3((unsigned)((Ni + 31) / 32), (unsigned)(kpad / 32)), 256, 0, st>>>(W, Ni, Ki, kpad, Wt);
    switch (act) {
        case BNN_ACT_SIGN: launch_realw_valu_lds<ACT_SIGN>(X, Wt, bias, Mi, Ki, kpad, Ni, Y, yw32, st); break;
        case BNN_ACT_HARDTANH: launch_realw_valu_lds<ACT_HARDTANH>(X, Wt, bias, Mi, Ki, kpad, Ni, Y, yw32, st); break;
        case BNN_ACT_SIGMOID: launch_realw_valu_lds<ACT_SIGMOID>(X, Wt, bias, Mi, Ki, kpad, Ni, Y, yw32, st); break;
        default: launch_realw_valu_lds<ACT_LINEAR>(X, Wt, bias, Mi, Ki, kpad, Ni, Y, yw32, st); break;
    }
    return launch_status();
}

// Real-input layers with binary weights on the int8 matrix cores as a tiled product (128 frames x 256 outputs per
// workgroup), inside bnn_forward for batches of 128 frames or more: Sign layers (three digit planes, exact bits: the
// outputs the filter cannot decide are listed and resolved by a second kernel) and the layer in front of the
// log-Softmax (four digit planes).  Scratch, all 256-byte aligned: digit planes, weight bytes, one record per frame,
// the list's counter, the list.
bool realx_i8_gemm_applies(const bnn_layer_desc& d, int64_t M) {
    return !d.x_is_binary && !d.w_is_real && d.K <= kSlabMaxK && M >= 128 &&
           (d.act == BNN_ACT_SIGN || d.act == BNN_ACT_LOGSOFTMAX);
}
struct I8GemmScratch {
    size_t planes, bytes, meta, undecided, total;
};
I8GemmScratch i8_gemm_scratch(int64_t M, int64_t K, int64_t N, int act) {
    const size_t kpad = (size_t)i8_kpad((int)K);
    const int digits = act == BNN_ACT_SIGN ? 3 : 4;
    I8GemmScratch s{};
    s.planes = 0;
    s.bytes = round_up((size_t)digits * (size_t)M * kpad, 256);
    s.meta = s.bytes + round_up((size_t)N * kpad, 256);
    s.undecided = s.meta + round_up((size_t)M * 16, 256);
    // Sign layers: a record per frame and tile of 256 outputs, room for 31 of them (the filter leaves about one output
    // in 250 undecided at K = 2048); what does not fit is summed by the lane that finds it
    const size_t tiles = (size_t)((N + kI8TileN - 1) / kI8TileN);
    s.total = s.undecided + (act == BNN_ACT_SIGN ? round_up((size_t)M * tiles * kUndecidedRecord, 256) : 0);
    return s;
}
template <int D>
int launch_realx_i8_gemm(const float* X, const void* Wp, const float* scale, const float* bias, int Mi, int Ki, int Ni, int w32,
                         void* Y, int yw32, char* mem, const I8GemmScratch& sc, hipStream_t st) {
    const int kpad = i8_kpad(Ki);
    int8_t* planes = reinterpret_cast<int8_t*>(mem + sc.planes);
    int8_t* bytes = reinterpret_cast<int8_t*>(mem + sc.bytes);
    void* meta = mem + sc.meta;
    unsigned char* undecided = reinterpret_cast<unsigned char*>(mem + sc.undecided);
    const int qbits = D == 3 ? slab_quant_bits(Ki) : kQuantBits4;
    if ((Ki & 3) == 0 && aligned(X, 16))
        realx_quantize_nat_kernel<D, true><<<dim3((Mi + 3) / 4), dim3(256), 0, st>>>(X, Mi, Ki, kpad, qbits, planes, meta);
    else
        realx_quantize_nat_kernel<D, false><<<dim3((Mi + 3) / 4), dim3(256), 0, st>>>(X, Mi, Ki, kpad, qbits, planes, meta);
    const int64_t eb = ((int64_t)Ni * (kpad / 16) + 255) / 256;
    bits_to_bytes_kernel<<<(unsigned)(eb < 16384 ? eb : 16384), 256, 0, st>>>(static_cast<const uint32_t*>(Wp), Ni, Ki, w32, kpad, bytes);
    static std::atomic<int> granted{0};   // more than 64 KB of LDS per workgroup has to be requested explicitly
    if (!granted.load()) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(realx_i8_gemm_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)i8_gemm_lds(D)) != hipSuccess) {
            (void)hipGetLastError();
            return BNN_EDEVICE;
        }
        granted.store(1);
    }
    const dim3 grid((unsigned)((Mi + kI8TileM - 1) / kI8TileM), (unsigned)((Ni + kI8TileN - 1) / kI8TileN));
    realx_i8_gemm_kernel<D><<<grid, kI8Threads, i8_gemm_lds(D), st>>>(planes, bytes, meta, X, static_cast<const uint32_t*>(Wp), scale, bias,
                                                                      Mi, Ki, kpad, Ni, w32, Y, yw32, D == 3 ? undecided : nullptr);
    if (D == 3) {
        const unsigned int rg = (unsigned int)((Mi + kResolveFrames - 1) / kResolveFrames);
        if ((Ki & 3) == 0 && aligned(X, 16))
            realx_resolve_rows_kernel<true><<<rg, kResolveThreads, 0, st>>>(X, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki, w32,
                                                                          undecided, (int)grid.y, static_cast<uint32_t*>(Y), yw32);
        else
            realx_resolve_rows_kernel<false><<<rg, kResolveThreads, 0, st>>>(X, static_cast<const uint32_t*>(Wp), scale, bias, Mi, Ki, w32,
                                                                           undecided, (int)grid.y, static_cast<uint32_t*>(Y), yw32);
    }
    return BNN_OK;
}
int run_realx_i8_gemm(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M, int64_t K, int64_t N, int wb,
                      int act, void* Y, void* scratch_mem, hipStream_t st) {
    const I8GemmScratch sc = i8_gemm_scratch(M, K, N, act);
    const int w32 = (int)row_w32(K, wb), yw32 = (int)row_w32(N, wb);
    int rc;
    if (act == BNN_ACT_SIGN) {
        rc = launch_realx_i8_gemm<3>(X, Wp, scale, bias, (int)M, (int)K, (int)N, w32, Y, yw32, static_cast<char*>(scratch_mem), sc, st);
    } else {
        rc = launch_realx_i8_gemm<4>(X, Wp, scale, bias, (int)M, (int)K, (int)N, w32, Y, 0, static_cast<char*>(scratch_mem), sc, st);
        if (rc == BNN_OK) launch_log_softmax(static_cast<float*>(Y), (int)M, (int)N, st);
    }
    return rc != BNN_OK ? rc : launch_status();
}

int check_chain(const bnn_layer_desc* L, int n_layers, int64_t M) {
    if (!L || n_layers <= 0) return BNN_EINVAL;
    if (M < 0 || M > kMaxDim) return BNN_ESHAPE;
    for (int l = 0; l < n_layers; ++l) {
        const bnn_layer_desc& d = L[l];
        if (!word_bits_ok(d.word_bits) || d.K <= 0 || d.N <= 0 || d.K > kMaxDim || d.N > kMaxN) return BNN_ESHAPE;
        if (d.act < BNN_ACT_LINEAR || d.act > BNN_ACT_SIGMOID) return BNN_EINVAL;
        if (d.w_is_real < 0 || d.w_is_real > 1 || (d.w_is_real && d.scale)) return BNN_EINVAL;
        if (d.x_is_binary < 0 || d.x_is_binary > 2) return BNN_EINVAL;
        if (!d.Wp) return BNN_EINVAL;
        if (l > 0) {
            const bnn_layer_desc& p = L[l - 1];
            if (d.K != p.N) return BNN_ESHAPE;
            if ((d.x_is_binary != 0) != (p.act == BNN_ACT_SIGN)) return BNN_ESHAPE;
            if (d.x_is_binary && d.word_bits != p.word_bits) return BNN_ESHAPE;
            if (p.act == BNN_ACT_LOGSOFTMAX) return BNN_ESHAPE;   // Softmax only closes a network (Alg. 2)
        }
    }
    return BNN_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------------ C ABI

BNN_EXPORT size_t bnn_packed_words(int64_t K, int word_bits) {
    if (K <= 0 || !word_bits_ok(word_bits)) return 0;
    return (size_t)words_per_row(K, word_bits);
}

BNN_EXPORT const char* bnn_status_string(int status) {
    switch (status) {
        case BNN_OK: return "ok";
        case BNN_EINVAL: return "invalid argument (null pointer, unknown activation or arm, overlapping buffers)";
        case BNN_ESHAPE: return "invalid shape (M < 0, K or N <= 0, word_bits not 32/64, or inconsistent layer chain)";
        case BNN_EALIGN: return "misaligned pointer";
        case BNN_EWORKSPACE: return "workspace missing or too small";
        case BNN_EDEVICE: return "HIP launch failed";
        default: return "unknown status";
    }
}

BNN_EXPORT int bnn_set_option(int option, int value) {
    switch (option) {
        case BNN_OPT_BINX_ARM:
            if (value != BNN_ARM_VALU_XOR && value != BNN_ARM_MFMA && value != BNN_ARM_MFMA_I8) return BNN_EINVAL;
            g_default_arm.store(value);
            return BNN_OK;
        case BNN_OPT_REALX_TM:
            if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8 && value != 16 && value != 32) return BNN_EINVAL;
            g_realx_tm.store(value);
            return BNN_OK;
        case BNN_OPT_STREAM_MAX_FRAMES:
            if (value < 0 || value > 4096) return BNN_EINVAL;
            g_stream_max_frames.store(value);
            return BNN_OK;
        case BNN_OPT_BINX_VALU_TM:
            if (value != 1 && value != 2 && value != 4 && value != 8 && value != 16 && value != 32) return BNN_EINVAL;
            g_binx_valu_tm.store(value);
            return BNN_OK;
        case BNN_OPT_MFMA_WM:
            if (value != 2 && value != 4) return BNN_EINVAL;
            g_mfma_wm.store(value);
            return BNN_OK;
        case BNN_OPT_MFMA_SHAPE:
            if (value != 0 && value != 16 && value != 32) return BNN_EINVAL;
            g_mfma_shape.store(value);
            return BNN_OK;
        case BNN_OPT_MFMA32_WM:
            if (value != 0 && value != 2 && value != 4) return BNN_EINVAL;
            g_mfma32_wm.store(value);
            return BNN_OK;
        case BNN_OPT_MFMA32_XCD_ORDER:
            if (value < 0 || value > 2) return BNN_EINVAL;
            g_mfma32_xcd_order.store(value);
            return BNN_OK;
        case BNN_OPT_REALX_F32_MFMA:
            if (value < 0 || value > 2) return BNN_EINVAL;
            g_realx_f32_mfma.store(value);
            return BNN_OK;
        case BNN_OPT_MFMA32_PIPELINE:
            if (value < 0 || value > 2) return BNN_EINVAL;
            g_mfma32_pipeline.store(value);
            return BNN_OK;
        case BNN_OPT_FUSED_LOGSOFTMAX:
            if (value != 0 && value != 1) return BNN_EINVAL;
            g_fused_softmax.store(value);
            return BNN_OK;
        case BNN_OPT_REALX_SIGN_MFMA:
            if (value < 0 || value > 2) return BNN_EINVAL;
            g_realx_sign_mfma.store(value);
            return BNN_OK;
        case BNN_OPT_COOPERATIVE:
            if (value != 0 && value != 1) return BNN_EINVAL;
            g_cooperative.store(value);
            return BNN_OK;
        case BNN_OPT_REALX_I8_LOGSOFTMAX:
            if (value < 0 || value > 2) return BNN_EINVAL;
            g_realx_i8_lsm.store(value);
            return BNN_OK;
        case BNN_OPT_REALW_SPLIT_LOGSOFTMAX:
            if (value < 0 || value > 2) return BNN_EINVAL;
            g_realw_split_lsm.store(value);
            return BNN_OK;
        case BNN_OPT_REALW_VALU_LDS:
            if (value != 0 && value != 1) return BNN_EINVAL;
            g_realw_valu_lds.store(value);
            return BNN_OK;
        case BNN_OPT_COOPERATIVE_SPIN:
            if (value < 1) return BNN_EINVAL;
            g_coop_spin.store(value);
            return BNN_OK;
        case BNN_OPT_MFMA32_SPLITK:
            if (value != 0 && value != 1) return BNN_EINVAL;
            g_mfma32_splitk.store(value);
            return BNN_OK;
        default: return BNN_EINVAL;
    }
}

BNN_EXPORT int bnn_cooperative_timeouts(uint64_t* count) {
    if (!count) return BNN_EINVAL;
    int dev = -1;
    unsigned char* base = coop_base(&dev);
    if (!base) return BNN_EDEVICE;
    unsigned int v = 0;
    if (hipDeviceSynchronize() != hipSuccess || hipMemcpy(&v, base, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return BNN_EDEVICE;
    }
    *count = v;
    return BNN_OK;
}

BNN_EXPORT int bnn_pack_weights(const float* W, int64_t N, int64_t K, int word_bits, void* Wp, float* scale_out,
                                void* stream) {
    if (!word_bits_ok(word_bits) || N <= 0 || K <= 0 || N > kMaxDim || K > kMaxDim) return BNN_ESHAPE;
    if (!W || !Wp) return BNN_EINVAL;
    if (!aligned(W, 4) || !aligned(Wp, word_bits / 8) || (scale_out && !aligned(scale_out, 4))) return BNN_EALIGN;
    const size_t wb = (size_t)N * K * 4, pb = (size_t)N * row_w32(K, word_bits) * 4;
    if (overlap(W, wb, Wp, pb) || (scale_out && (overlap(W, wb, scale_out, 4) || overlap(Wp, pb, scale_out, 4))))
        return BNN_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int rc = run_pack(W, N, K, word_bits, Wp, st);
    if (rc != BNN_OK) return rc;
    if (scale_out) {
        mean_abs_kernel<<<dim3(1), dim3(1024), 0, st>>>(W, N * K, scale_out);
        return launch_status();
    }
    return BNN_OK;
}

BNN_EXPORT int bnn_pack_activations(const float* X, int64_t M, int64_t K, int word_bits, void* Xp, void* stream) {
    if (!word_bits_ok(word_bits) || M < 0 || K <= 0 || M > kMaxDim || K > kMaxDim) return BNN_ESHAPE;
    if (M == 0) return BNN_OK;
    if (!X || !Xp) return BNN_EINVAL;
    if (!aligned(X, 4) || !aligned(Xp, word_bits / 8)) return BNN_EALIGN;
    if (overlap(X, (size_t)M * K * 4, Xp, (size_t)M * row_w32(K, word_bits) * 4)) return BNN_EINVAL;
    return run_pack(X, M, K, word_bits, Xp, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_layer_binw_realx(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M,
                                    int64_t K, int64_t N, int act, int word_bits, void* Y, void* stream) {
    const int rc = check_layer_args(X, Wp, M, K, N, act, word_bits, Y, false);
    if (rc != BNN_OK) return rc;
    return run_realx(X, Wp, scale, bias, M, K, N, act, word_bits, Y, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_layer_binw_binx_arm(const void* Xp, const void* Wp, const float* scale, const float* bias, int64_t M,
                                       int64_t K, int64_t N, int act, int word_bits, void* Y, int arm, void* stream) {
    if (arm != BNN_ARM_AUTO && arm != BNN_ARM_VALU_XOR && arm != BNN_ARM_MFMA && arm != BNN_ARM_MFMA_I8) return BNN_EINVAL;
    const int rc = check_layer_args(Xp, Wp, M, K, N, act, word_bits, Y, true);
    if (rc != BNN_OK) return rc;
    return run_binx(Xp, Wp, scale, bias, M, K, N, act, word_bits, Y, arm, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_layer_binw_binx01(const void* Xp, const void* Wp, const float* scale, const float* bias, int64_t M,
                                     int64_t K, int64_t N, int act, int word_bits, void* Y, void* stream) {
    const int rc = check_layer_args(Xp, Wp, M, K, N, act, word_bits, Y, true);
    if (rc != BNN_OK) return rc;
    return run_binx(Xp, Wp, scale, bias, M, K, N, act, word_bits, Y, BNN_ARM_MFMA, static_cast<hipStream_t>(stream), true);
}

BNN_EXPORT int bnn_layer_binw_binx(const void* Xp, const void* Wp, const float* scale, const float* bias, int64_t M,
                                   int64_t K, int64_t N, int act, int word_bits, void* Y, void* stream) {
    return bnn_layer_binw_binx_arm(Xp, Wp, scale, bias, M, K, N, act, word_bits, Y, BNN_ARM_AUTO, stream);
}

BNN_EXPORT int bnn_layer_realw(const float* X, const float* W, const float* bias, int64_t M, int64_t K, int64_t N, int act,
                               int word_bits, void* Y, void* stream) {
    const int rc = check_layer_args(X, W, M, K, N, act, word_bits, Y, false, true);
    if (rc != BNN_OK) return rc;
    return run_realw(X, W, bias, M, K, N, act, word_bits, Y, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_unpack_activations(const void* Xp, int64_t M, int64_t K, int word_bits, int zero_one, float* X,
                                      void* stream) {
    if (!word_bits_ok(word_bits) || M < 0 || K <= 0 || M > kMaxDim || K > kMaxDim) return BNN_ESHAPE;
    if (zero_one < 0 || zero_one > 1) return BNN_EINVAL;
    if (M == 0) return BNN_OK;
    if (!Xp || !X) return BNN_EINVAL;
    if (!aligned(Xp, word_bits / 8) || !aligned(X, 4)) return BNN_EALIGN;
    if (overlap(Xp, (size_t)M * row_w32(K, word_bits) * 4, X, (size_t)M * K * 4)) return BNN_EINVAL;
    return run_unpack(Xp, M, K, word_bits, zero_one, X, static_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------------------------------------ training side

namespace {
unsigned elementwise_blocks(int64_t count) {
    const int64_t b = (count + 255) / 256;
    return (unsigned)(b < 65536 ? (b > 0 ? b : 1) : 65536);
}
bool dims_ok(int64_t a, int64_t b) { return a > 0 && b > 0 && a <= kMaxDim && b <= kMaxDim; }
}  // namespace

BNN_EXPORT int bnn_pack_weights_transposed(const float* W, int64_t N, int64_t K, int word_bits, void* WpT, void* stream) {
    if (!word_bits_ok(word_bits) || !dims_ok(N, K)) return BNN_ESHAPE;
    if (!W || !WpT) return BNN_EINVAL;
    if (!aligned(W, 4) || !aligned(WpT, word_bits / 8)) return BNN_EALIGN;
    const int w32t = (int)row_w32(N, word_bits);
    if (overlap(W, (size_t)N * K * 4, WpT, (size_t)K * w32t * 4)) return BNN_EINVAL;
    const dim3 grid((unsigned)((K + 63) / 64), (unsigned)((N + 63) / 64));
    pack_sign_transposed_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(W, (int)N, (int)K, w32t,
                                                                                     static_cast<uint32_t*>(WpT));
    return launch_status();
}

BNN_EXPORT int bnn_transpose_f32(const float* A, int64_t R, int64_t C, float* out, void* stream) {
    if (!dims_ok(R, C)) return BNN_ESHAPE;
    if (!A || !out) return BNN_EINVAL;
    if (!aligned(A, 4) || !aligned(out, 4)) return BNN_EALIGN;
    if (overlap(A, (size_t)R * C * 4, out, (size_t)R * C * 4)) return BNN_EINVAL;
    const dim3 grid((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64));
    transpose_f32_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(A, (int)R, (int)C, out);
    return launch_status();
}

BNN_EXPORT int bnn_softmax_xent_grad(const float* logp, const int32_t* labels, int64_t M, int64_t N, float* g, void* stream) {
    if (M < 0 || N <= 0 || M > kMaxDim || N > kMaxDim) return BNN_ESHAPE;
    if (M == 0) return BNN_OK;
    if (!logp || !labels || !g) return BNN_EINVAL;
    if (!aligned(logp, 4) || !aligned(labels, 4) || !aligned(g, 4)) return BNN_EALIGN;
    softmax_xent_grad_kernel<<<elementwise_blocks(M * N), 256, 0, static_cast<hipStream_t>(stream)>>>(logp, labels, M, (int)N, g);
    return launch_status();
}

BNN_EXPORT int bnn_mask_grad(const float* g_h, const float* hhat, int64_t count, float k, float* g_hhat, void* stream) {
    if (count < 0) return BNN_ESHAPE;
    if (!(k > 0.0f)) return BNN_EINVAL;
    if (count == 0) return BNN_OK;
    if (!g_h || !hhat || !g_hhat) return BNN_EINVAL;
    if (!aligned(g_h, 4) || !aligned(hhat, 4) || !aligned(g_hhat, 4)) return BNN_EALIGN;
    mask_grad_kernel<<<elementwise_blocks(count), 256, 0, static_cast<hipStream_t>(stream)>>>(g_h, hhat, count, k, g_hhat);
    return launch_status();
}

BNN_EXPORT int bnn_sigmoid_grad(const float* g_h, const float* h, int64_t count, float* g_hhat, void* stream) {
    if (count < 0) return BNN_ESHAPE;
    if (count == 0) return BNN_OK;
    if (!g_h || !h || !g_hhat) return BNN_EINVAL;
    if (!aligned(g_h, 4) || !aligned(h, 4) || !aligned(g_hhat, 4)) return BNN_EALIGN;
    sigmoid_grad_kernel<<<elementwise_blocks(count), 256, 0, static_cast<hipStream_t>(stream)>>>(g_h, h, count, g_hhat);
    return launch_status();
}

BNN_EXPORT size_t bnn_layer_binw_realx_i8_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M <= 0 || K <= 0 || N <= 0 || M > kMaxDim || K > kSlabMaxK || N > kMaxN) return 0;
    return i8_gemm_scratch(M, K, N, BNN_ACT_LINEAR).total;
}

BNN_EXPORT int bnn_layer_binw_realx_i8(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M,
                                       int64_t K, int64_t N, int word_bits, float* Y, void* workspace, size_t workspace_bytes,
                                       void* stream) {
    const int rc = check_layer_args(X, Wp, M, K, N, BNN_ACT_LINEAR, word_bits, Y, false);
    if (rc != BNN_OK) return rc;
    if (K > kSlabMaxK) return BNN_ESHAPE;
    if (M == 0) return BNN_OK;
    const I8GemmScratch sc = i8_gemm_scratch(M, K, N, BNN_ACT_LINEAR);
    if (!workspace || workspace_bytes < sc.total) return BNN_EWORKSPACE;
    if (!aligned(workspace, 256)) return BNN_EALIGN;
    const size_t yb = (size_t)M * N * 4;
    if (overlap(workspace, sc.total, Y, yb) || overlap(workspace, sc.total, X, (size_t)M * K * 4) ||
        overlap(workspace, sc.total, Wp, (size_t)N * row_w32(K, word_bits) * 4))
        return BNN_EINVAL;
    const int lrc = launch_realx_i8_gemm<4>(X, Wp, scale, bias, (int)M, (int)K, (int)N, (int)row_w32(K, word_bits), Y, 0,
                                            static_cast<char*>(workspace), sc, static_cast<hipStream_t>(stream));
    return lrc != BNN_OK ? lrc : launch_status();
}

BNN_EXPORT int bnn_backward_input_binw(const float* g_hhat, const void* WpT, int64_t M, int64_t N, int64_t K, int word_bits,
                                       float* g_h, void* stream) {
    // the forward layer with the roles exchanged: "inputs" are the N gradients of a frame, "outputs" the K inputs
    const int rc = check_layer_args(g_hhat, WpT, M, N, K, BNN_ACT_LINEAR, word_bits, g_h, false);
    if (rc != BNN_OK) return rc;
    return run_realx(g_hhat, WpT, nullptr, nullptr, M, N, K, BNN_ACT_LINEAR, word_bits, g_h, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_backward_input_realw(const float* g_hhat, const float* Wt, int64_t M, int64_t N, int64_t K, float* g_h,
                                        void* stream) {
    const int rc = check_layer_args(g_hhat, Wt, M, N, K, BNN_ACT_LINEAR, 32, g_h, false, true);
    if (rc != BNN_OK) return rc;
    return run_realw(g_hhat, Wt, nullptr, M, N, K, BNN_ACT_LINEAR, 32, g_h, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_backward_weight(const float* g_hhat_t, const float* h_t, int64_t N, int64_t K, int64_t M, float* g_w,
                                   void* stream) {
    // rows of the "frame" operand are the N outputs, the sum runs over the M frames, "outputs" are the K inputs
    if (M <= 0) return BNN_ESHAPE;
    const int rc = check_layer_args(g_hhat_t, h_t, N, M, K, BNN_ACT_LINEAR, 32, g_w, false, true);
    if (rc != BNN_OK) return rc;
    return run_realw(g_hhat_t, h_t, nullptr, N, M, K, BNN_ACT_LINEAR, 32, g_w, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_backward_weight_binh(const float* g_hhat_t, const void* HpT, int64_t N, int64_t K, int64_t M, int word_bits,
                                        float* g_w, void* stream) {
    if (M <= 0) return BNN_ESHAPE;
    const int rc = check_layer_args(g_hhat_t, HpT, N, M, K, BNN_ACT_LINEAR, word_bits, g_w, false);
    if (rc != BNN_OK) return rc;
    return run_realx(g_hhat_t, HpT, nullptr, nullptr, N, M, K, BNN_ACT_LINEAR, word_bits, g_w, static_cast<hipStream_t>(stream));
}

BNN_EXPORT int bnn_bias_grad(const float* g_hhat, int64_t M, int64_t N, float* g_r, void* stream) {
    if (M < 0 || N <= 0 || M > kMaxDim || N > kMaxDim) return BNN_ESHAPE;
    if (!g_hhat || !g_r) return BNN_EINVAL;
    if (!aligned(g_hhat, 4) || !aligned(g_r, 4)) return BNN_EALIGN;
    if (overlap(g_hhat, (size_t)M * N * 4, g_r, (size_t)N * 4)) return BNN_EINVAL;
    colsum_kernel<<<(unsigned)((N + 63) / 64), 64, 0, static_cast<hipStream_t>(stream)>>>(g_hhat, (int)M, (int)N, g_r);
    return launch_status();
}

BNN_EXPORT int bnn_update_clip(float* w, const float* g, int64_t count, float eta, int clip, void* stream) {
    if (count < 0) return BNN_ESHAPE;
    if (clip < 0 || clip > 1) return BNN_EINVAL;
    if (count == 0) return BNN_OK;
    if (!w || !g) return BNN_EINVAL;
    if (!aligned(w, 4) || !aligned(g, 4)) return BNN_EALIGN;
    if (overlap(w, (size_t)count * 4, g, (size_t)count * 4)) return BNN_EINVAL;
    update_clip_kernel<<<elementwise_blocks(count), 256, 0, static_cast<hipStream_t>(stream)>>>(w, g, count, eta, clip);
    return launch_status();
}

BNN_EXPORT int bnn_grad_norm_clip(float* g, int64_t count, float alpha, void* workspace, float* norm_out, void* stream) {
    if (count < 0) return BNN_ESHAPE;
    if (!(alpha > 0.0f)) return BNN_EINVAL;
    if (!g || !workspace || !norm_out) return BNN_EINVAL;
    if (!aligned(g, 4) || !aligned(workspace, 8) || !aligned(norm_out, 4)) return BNN_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    double* partial = static_cast<double*>(workspace);
    sumsq_partial_kernel<<<kSumsqBlocks, 256, 0, st>>>(g, count, partial);
    sumsq_final_kernel<<<1, 256, 0, st>>>(partial, norm_out);
    if (count > 0) scale_if_above_kernel<<<elementwise_blocks(count), 256, 0, st>>>(g, count, alpha, norm_out);
    return launch_status();
}

BNN_EXPORT int bnn_subtract_log_prior(float* logp, const float* log_prior, int64_t M, int64_t N, void* stream) {
    if (M < 0 || N <= 0 || M > kMaxDim || N > kMaxN) return BNN_ESHAPE;
    if (M == 0) return BNN_OK;
    if (!logp || !log_prior) return BNN_EINVAL;
    if (!aligned(logp, 4) || !aligned(log_prior, 4)) return BNN_EALIGN;
    if (overlap(logp, (size_t)M * (size_t)N * 4, log_prior, (size_t)N * 4)) return BNN_EINVAL;
    subtract_log_prior_kernel<<<elementwise_blocks(M * N), 256, 0, static_cast<hipStream_t>(stream)>>>(logp, log_prior, M, (int)N);
    return launch_status();
}

BNN_EXPORT int bnn_semi_stochastic_binarize(float* w, const float* u, int64_t count, void* stream) {
    if (count < 0) return BNN_ESHAPE;
    if (count == 0) return BNN_OK;
    if (!w || !u) return BNN_EINVAL;
    if (!aligned(w, 4) || !aligned(u, 4)) return BNN_EALIGN;
    if (overlap(w, (size_t)count * 4, u, (size_t)count * 4)) return BNN_EINVAL;
    semi_stochastic_kernel<<<elementwise_blocks(count), 256, 0, static_cast<hipStream_t>(stream)>>>(w, u, count);
    return launch_status();
}

// Workspace layout of bnn_forward: two ping-pong buffers of `half` bytes, then `unpacked` bytes for the fp32 copy of
// the bits that a real-weight layer reads, or for the digit planes of a real-input Sign layer (whichever is larger).
struct ForwardWorkspace {
    size_t half, unpacked;
};
// `roomy`: with the scratch of the tiled matrix-core products (the weight bytes and the list of realx_i8_gemm, the bf16
// planes of a Softmax layer with real weights); without it those layers run on the kernels that need less or none
static ForwardWorkspace forward_workspace(const bnn_layer_desc* layers, int n_layers, int64_t M, bool roomy = true) {
    size_t biggest = 0, unpacked = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (l + 1 < n_layers) {
            const size_t b = out_bytes(M, layers[l].N, layers[l].act, layers[l].word_bits);
            if (b > biggest) biggest = b;
        }
        if (layers[l].w_is_real) {
            // unpacked binary input first, then the bf16 planes of both operands of a Softmax layer with real weights, or
            // the transposed weights of another layer with real weights
            size_t b = layers[l].x_is_binary ? round_up((size_t)M * (size_t)layers[l].K * 4, 256) : 0;
            if (roomy && realw_split_lsm_applies(layers[l], M)) b += realw_split_lsm_bytes(M, layers[l].K, layers[l].N);
            if (roomy && realw_valu_lds_applies(layers[l], M)) b += realw_valu_lds_bytes(layers[l].K, layers[l].N);
            if (b > unpacked) unpacked = b;
        }
        if (realx_i8_lsm_applies(layers[l], M)) {
            const size_t b = realx_i8_lsm_bytes(M, layers[l].K);
            if (b > unpacked) unpacked = b;
        }
        if (roomy && realx_i8_gemm_applies(layers[l], M) && !(l == 0 && realx_sign_mfma_applies(layers[l]))) {
            const size_t b = i8_gemm_scratch(M, layers[l].K, layers[l].N, layers[l].act).total;
            if (b > unpacked) unpacked = b;
        }
        // digit planes of a real-input Sign layer that the first-layer kernel does not take (same region: one layer at a time)
        if (realx_sign_slab_applies(layers[l]) && !(l == 0 && realx_sign_mfma_applies(layers[l]))) {
            const size_t b = realx_sign_slab_bytes(M, layers[l].K);
            if (b > unpacked) unpacked = b;
        }
    }
    return {round_up(biggest, 256), round_up(unpacked, 256)};
}

BNN_EXPORT size_t bnn_forward_workspace_bytes(const bnn_layer_desc* layers, int n_layers, int64_t M) {
    if (check_chain(layers, n_layers, M) != BNN_OK) return 0;
    const ForwardWorkspace ws = forward_workspace(layers, n_layers, M);
    return 2 * ws.half + ws.unpacked;
}

// Scratch of bnn_forward_static: a fixed array in the library's device image (every GPU the library runs on holds its
// own copy at its own address until the process ends).  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and copies get the device address that call returns.
constexpr size_t kStaticScratchBytes = (size_t)BNN_FORWARD_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}
}  // namespace

static int forward_run(const bnn_layer_desc* layers, int n_layers, const void* X, int64_t M, void* out, void* workspace,
                       size_t workspace_bytes, void* stream, bool roomy);

BNN_EXPORT int bnn_forward_static(const bnn_layer_desc* layers, int n_layers, const void* X, int64_t M, void* out,
                                  void* stream) {
    const int rc = check_chain(layers, n_layers, M);
    if (rc != BNN_OK) return rc;
    if (M == 0) return BNN_OK;
    // The scratch of the tiled matrix-core products (a byte per weight of a real-input layer, six bytes per weight of a
    // Softmax layer with real weights) is left out when it does not fit the array: those layers then run on the kernels
    // bnn_forward uses with these products switched off.
    bool roomy = true;
    ForwardWorkspace ws = forward_workspace(layers, n_layers, M, true);
    if (2 * ws.half + ws.unpacked > kStaticScratchBytes) {
        roomy = false;
        ws = forward_workspace(layers, n_layers, M, false);
    }
    const size_t need = 2 * ws.half + ws.unpacked;
    if (need > kStaticScratchBytes) return BNN_EWORKSPACE;
    void* mem = nullptr;
    if (need) {
        mem = static_scratch();
        if (!mem) return BNN_EDEVICE;
    }
    return forward_run(layers, n_layers, X, M, out, mem, need, stream, roomy);
}

BNN_EXPORT int bnn_forward(const bnn_layer_desc* layers, int n_layers, const void* X, int64_t M, void* out,
                           void* workspace, size_t workspace_bytes, void* stream) {
    return forward_run(layers, n_layers, X, M, out, workspace, workspace_bytes, stream, true);
}

static int forward_run(const bnn_layer_desc* layers, int n_layers, const void* X, int64_t M, void* out, void* workspace,
                       size_t workspace_bytes, void* stream, bool roomy) {
    int rc = check_chain(layers, n_layers, M);
    if (rc != BNN_OK) return rc;
    if (M == 0) return BNN_OK;
    if (!X || !out) return BNN_EINVAL;
    const ForwardWorkspace ws = forward_workspace(layers, n_layers, M, roomy);
    const size_t need = 2 * ws.half + ws.unpacked;
    if (need && (!workspace || workspace_bytes < need)) return BNN_EWORKSPACE;
    if (need && !aligned(workspace, 256)) return BNN_EALIGN;
    // Check every layer's arguments before anything is enqueued.
    char* buf[2] = {static_cast<char*>(workspace), static_cast<char*>(workspace) + ws.half};
    float* unpacked = reinterpret_cast<float*>(static_cast<char*>(workspace) + 2 * ws.half);
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int pass = 0; pass < 2; ++pass) {
        const void* in = X;
        for (int l = 0; l < n_layers; ++l) {
            const bnn_layer_desc& d = layers[l];
            void* o = (l == n_layers - 1) ? out : static_cast<void*>(buf[l & 1]);
            if (pass == 0) {
                if (d.w_is_real && d.x_is_binary) {
                    if (!aligned(in, d.word_bits / 8)) return BNN_EALIGN;
                    rc = check_layer_args(unpacked, d.Wp, M, d.K, d.N, d.act, d.word_bits, o, false, true);
                } else {
                    rc = check_layer_args(in, d.Wp, M, d.K, d.N, d.act, d.word_bits, o, d.x_is_binary != 0, d.w_is_real != 0);
                }
            } else if (d.w_is_real) {
                const float* xin = static_cast<const float*>(in);
                char* planes = reinterpret_cast<char*>(unpacked);
                if (d.x_is_binary) {
                    rc = run_unpack(in, M, d.K, d.word_bits, d.x_is_binary == 2, unpacked, st);
                    if (rc != BNN_OK) return rc;
                    xin = unpacked;
                    planes += round_up((size_t)M * (size_t)d.K * 4, 256);
                }
                if (roomy && realw_split_lsm_applies(d, M) && g_realw_split_lsm.load() && g_realx_f32_mfma.load() != 2 &&
                    M > g_stream_max_frames.load())
                    rc = run_realw_split_lsm(xin, static_cast<const float*>(d.Wp), d.bias, M, d.K, d.N,
                                             static_cast<float*>(o), planes, st);
                else if (roomy && realw_valu_lds_applies(d, M) && g_realw_valu_lds.load() && M > g_stream_max_frames.load() &&
                         !(d.act != BNN_ACT_SIGN && g_realx_f32_mfma.load() == 1) && aligned(xin, 16))
                    rc = run_realw_valu_lds(xin, static_cast<const float*>(d.Wp), d.bias, M, d.K, d.N, d.act, d.word_bits, o,
                                            planes, st);
                else
                    rc = run_realw(xin, static_cast<const float*>(d.Wp), d.bias, M, d.K, d.N, d.act, d.word_bits, o, st);
            } else if (d.x_is_binary) {
                rc = run_binx(in, d.Wp, d.scale, d.bias, M, d.K, d.N, d.act, d.word_bits, o, BNN_ARM_AUTO, st,
                              d.x_is_binary == 2);
            } else if (l == 0 && realx_sign_mfma_applies(d) && g_realx_sign_mfma.load() && M > g_stream_max_frames.load()) {
                rc = run_realx_sign_mfma(static_cast<const float*>(in), d.Wp, d.scale, d.bias, M, d.K, d.N, d.word_bits,
                                         o, st);
            } else if (roomy && realx_i8_gemm_applies(d, M) && M > g_stream_max_frames.load() &&
                       (d.act == BNN_ACT_SIGN ? g_realx_sign_mfma.load() == 1
                                              : (g_realx_i8_lsm.load() == 1 && g_realx_f32_mfma.load() != 2))) {
                rc = run_realx_i8_gemm(static_cast<const float*>(in), d.Wp, d.scale, d.bias, M, d.K, d.N, d.word_bits, d.act, o,
                                       unpacked, st);
            } else if (realx_i8_lsm_applies(d, M) && g_realx_i8_lsm.load() && g_realx_f32_mfma.load() != 2 &&
                       M > g_stream_max_frames.load()) {
                rc = run_realx_i8_lsm(static_cast<const float*>(in), d.Wp, d.scale, d.bias, M, d.K, d.N, d.word_bits,
                                      static_cast<float*>(o), unpacked, st);
            } else if (realx_sign_slab_applies(d) && g_realx_sign_mfma.load() && M > g_stream_max_frames.load()) {
                rc = run_realx_sign_slab(static_cast<const float*>(in), d.Wp, d.scale, d.bias, M, d.K, d.N, d.word_bits, o,
                                         unpacked, st);
            } else {
                rc = run_realx(static_cast<const float*>(in), d.Wp, d.scale, d.bias, M, d.K, d.N, d.act, d.word_bits, o,
                               st);
            }
            if (rc != BNN_OK) return rc;
            in = o;
        }
    }
    return BNN_OK;
}
