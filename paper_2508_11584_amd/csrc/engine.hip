// The engine behind the C ABI of vpe.h: device memory plan, weight upload and re-layout,
// the encoder and head launch sequences, and the frame scheduler (feature-slot ring guarded
// by HIP events, per-head streams and rate dividers, optional HIP-graph replay).
//
// Mapping to the paper (Sec. "System architecture"): vpe_encode is the foundation module,
// the slot ring is its "middle buffer" (a circular GPU buffer that is overwritten oldest
// first), vpe_run_head is a head module reading that buffer by reference, and every_n is the
// per-head frequency control.  The paper's one-process-per-module + MPS design is replaced by
// one process with one HIP stream per module.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "kernels.h"
#include "vpe.h"

using namespace vpe;

// Scratch for vpe_run_head_static: callers that may not allocate (and may not trigger an allocation inside the
// library) get their head's intermediate buffers from this array instead of from an engine workspace.  One copy
// per GPU the library is loaded on, held until the process ends; every call on a GPU shares it.
constexpr uint64_t STATIC_SCRATCH_BYTES = 8ull << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_create_error;

// Device address of `scratch` on each GPU (the array's name is a host-side stand-in, not a device address; each
// GPU has its own copy at its own address).  Looked up once per device, with that device current.
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

hipError_t static_scratch(int device, void** out) {
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t rc = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (rc != hipSuccess) return rc;
        if (!ptr || ((uintptr_t)ptr & 255)) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

constexpr int KPATCH = 588;      // 3 * 14 * 14
constexpr int KPATCH_PAD = 640;  // next multiple of the k-tile
constexpr int NPAD = 256;        // weight rows are padded to the widest GEMM tile
constexpr int MAX_LANES = 4;
constexpr int HW_QUEUES = 4;      // hardware queues a process gets by default

struct Bump {
    char* base = nullptr;  // null: only count
    uint64_t off = 0;
    void* take(uint64_t bytes) {
        off = (uint64_t)rup((int64_t)off, 256);
        void* p = base ? base + off : nullptr;
        off += bytes;
        return p;
    }
};

struct BlockW {
    // The two in-block LayerNorms are folded into the GEMMs that consume them: qkv_w / fc1_w are scaled by the
    // LayerNorm gain along k, qkv_b / fc1_b hold b + beta W, and qkv_s / fc1_s the column sums of the scaled,
    // rounded weights (see GemmArgs::ln_stats).  ln1_* / ln2_* are only kept for the upload.
    float *ln1_g, *ln1_b, *qkv_b, *qkv_s, *proj_b, *ls1, *ln2_g, *ln2_b, *fc1_b, *fc1_s, *fc2_b, *ls2;
    void *qkv_w, *proj_w, *fc1_w, *fc2_w;
};

struct ConvW { void* w = nullptr; float* b = nullptr; };

// State of a full DPT head (reassemble -> fusion with residual convolution units -> output convolutions).
// Maps are pixel-major with the channel count rounded up to 64 (`ocp`, `hp`); the padding channels are zero
// (the workspace is cleared at creation and nothing writes them) and meet zero weight columns.
struct Dpt {
    int F = 0, oc[4] = {}, ocp[4] = {}, hh[4] = {}, ww[4] = {}, hp = 0;   // level i: oc[i] channels on an hh[i] x ww[i] grid
    // levels 0 and 1: tap projection and transposed convolution (kernel = stride s) composed into s*s matrices
    // [oc][D], one per position (dy, dx) inside the s x s block, with their biases
    void* up_w[2] = {};
    float* up_b[2] = {};
    ConvW proj[2];                 // taps 2 and 3
    ConvW down3, rn[4];
    ConvW fa1[4], fa2[4], fb1[4], fb2[4], fout[4];   // per level k: residual units a (k < 3) and b, output 1x1
    ConvW head1, head2;
    float* head3_w = nullptr;      // [64], 32 in use
    float head3_b = 0.0f;
    // activations
    void* R[4] = {};               // reassembled maps [n_i][ocp_i]
    void *P3 = nullptr, *G3 = nullptr;
    float* L[4] = {};              // l_i in fp32 (residual operand)
    void* Lr[4] = {};              // ReLU(l_i) in the engine dtype (convolution operand)
    void *t = nullptr, *sr = nullptr, *y = nullptr, *c = nullptr, *path0 = nullptr, *o1 = nullptr, *u = nullptr;
    float *s = nullptr, *path[2] = {}, *dpart = nullptr;
    void* ty[5] = {};              // aligned-corner tap tables of the five resizes (rows, columns)
    void* tx[5] = {};
    int rh[5] = {}, rw[5] = {};    // their output sizes
};

// Intermediate buffers of a seg / det / DPT-lite head run (neither its input, the feature slot, nor its outputs):
// normally part of the engine's workspace, or carved out of the library's static device array for
// vpe_run_head_static.  Every element a run reads is written earlier in the same run; nothing relies on old contents.
struct HeadScratch {
    void* tower = nullptr;         // det [B P][2 ch]
    void* p[4] = {};               // depth: tap projections [B P][ch]
    void *z = nullptr, *r = nullptr;   // depth: stage input / convolution output [B 64 P][ch], reused across stages
    float* d8 = nullptr;           // depth: [pixel][ch / 64] partial 1-channel projections on the 8x grid
};

struct Head {
    int kind = 0, classes = 0, ch = 0, every_n = 1;
    Dpt dpt;
    HeadScratch sc;
    // weights
    void* w0 = nullptr;            // seg: [C][D]; det: towers [2ch][9D]; depth: unused
    float* b0 = nullptr;
    void* w1 = nullptr;            // det: block-diagonal [classes + 4][2 ch]
    float* b1 = nullptr;
    void* proj_w[4] = {};          // depth
    float* proj_b[4] = {};
    void* fuse_w[4] = {};
    float* fuse_b[4] = {};
    float* out_w = nullptr;
    float out_b = 0.0f;
    // activations / outputs
    float* logits = nullptr;       // seg [B P][C]; det [B P][classes + 4]
    uint8_t* classmap = nullptr;
    float* depth = nullptr;
    // scheduling
    hipStream_t stream = nullptr;     // one of the engine's head streams (shared when heads outnumber them)
    hipEvent_t last_done = nullptr;   // completion of the most recent run (any slot)
    hipEvent_t t_begin = nullptr, t_end = nullptr;   // around the most recent run (engines created with VPE_FLAG_TIMING)
    bool ran = false;
    int64_t runs = 0, skips = 0;
    double period = 0.0;              // 1 / max_hz, 0 = no limit in Hz
    double due = 0.0;                 // frame time from which the next run is allowed
    bool due_set = false;
    // lossy-freshness bookkeeping
    int64_t seen = -1;                // newest frame this head has been asked about
    int64_t last_run_frame = -1;
    int64_t missed = 0;               // frames passed over because a newer one was taken
    int64_t overflow = 0;             // frames overwritten in the ring before the head was asked about them
    int64_t busy = 0;                 // vpe_run_head_latest calls turned away because the previous run was still going
    std::vector<hipGraphExec_t> graphs;   // per slot
};

}  // namespace

struct vpe_engine {
    vpe_backbone_cfg cfg{};
    bool bf = true, host_only = false, graphs = false, owns_ws = false, timing = false;
    int last_lane = -1;                  // lane of the most recent encode
    int device = -1;                     // the GPU the engine lives on
    void* static_ptr = nullptr;          // that GPU's copy of the library's static scratch array
    int D = 0, L = 0, nh = 0, Mh = 0, F = 0, R = 0, B = 0, H = 0, W = 0, gh = 0, gw = 0, P = 0, N = 0, T = 0;
    int npad = 0, esz = 2, S = 1;
    char* ws = nullptr;
    uint64_t ws_bytes = 0;
    // backbone weights
    void* patch_w = nullptr;
    float *patch_b = nullptr, *special = nullptr, *pos = nullptr, *norm_g = nullptr, *norm_b = nullptr;
    std::vector<BlockW> blk;
    // encoder scratch
    void* zeros = nullptr;               // 256 bytes that stay zero (padding taps of the 3x3 convolutions)
    float* lev0 = nullptr;               // [T] level of a fresh frame's rows: mean over the width of bias + positional row
    // Encoder lanes: `lanes` complete scratch sets, each with its own stream.  Frame f is encoded on lane
    // f % lanes, so with two lanes the encoder passes of consecutive frames overlap on the GPU (the ViT-S
    // kernels are too small to fill 256 CUs on their own); results per frame are unchanged.
    struct Lane {
        // x: fp32 residual stream; u: its copy in the engine dtype (the A operand of the LayerNorm-folded
        // GEMMs; unused by fp32 engines, which read x); stats: per row and 64-column group (mean, sum of squared deviations) of x
        void *apatch = nullptr, *u = nullptr, *qk = nullptr, *vt = nullptr, *att = nullptr, *hid = nullptr;
        float *x = nullptr, *stats = nullptr;
        float* lev[2] = {nullptr, nullptr};   // [T] row levels the copy u is stored against, alternating (see ln_gemm)
        hipStream_t stream = nullptr;
        hipEvent_t done = nullptr;      // completion of the lane's most recent encode
        hipEvent_t t_begin = nullptr, t_end = nullptr;   // around it (engines created with VPE_FLAG_TIMING)
        bool used = false;
    };
    int lanes = 1;
    Lane lane[MAX_LANES];
    // ring
    std::vector<void*> feat;             // [S][4]
    std::vector<int64_t> slot_frame;     // frame held by each slot, -1 = none
    std::vector<double> slot_time;       // its capture time, NaN = none given
    double last_time = 0.0;
    bool have_time = false;
    bool wall_clock = false;             // frames without a time are stamped with the host's steady clock
    std::chrono::steady_clock::time_point t0;
    std::vector<hipEvent_t> ready;       // [S]
    std::vector<hipEvent_t> done;        // [S][n_heads]
    std::vector<char> done_set;          // [S][n_heads]
    std::vector<hipGraphExec_t> enc_graphs;   // [S][lanes]
    std::vector<Head> heads;
    std::vector<hipStream_t> head_streams;
    int64_t frames = 0;
    std::string err;

    int fail(int code, const std::string& m) { err = m; return code; }
};

namespace {

#define HIPCHK(e, call)                                                                      \
    do {                                                                                     \
        hipError_t err__ = (call);                                                           \
        if (err__ != hipSuccess)                                                             \
            return (e)->fail(VPE_EHIP, std::string(#call) + ": " + hipGetErrorString(err__)); \
    } while (0)

int64_t backbone_floats(const vpe_backbone_cfg& c) {
    const int64_t D = c.dim, P = (int64_t)(c.img_h / 14) * (c.img_w / 14);
    const int64_t F = (int64_t)c.mlp_hidden * (c.mlp_kind == VPE_MLP_SWIGLU ? 2 : 1);
    int64_t n = D * KPATCH + D + D + (int64_t)c.registers * D + (1 + P) * D;
    n += c.depth * (2 * D + D * 3 * D + 3 * D + D * D + D + D + 2 * D + D * F + F + c.mlp_hidden * D + D + D);
    return n + 2 * D;
}

int64_t head_floats(const vpe_backbone_cfg& c, const vpe_head_cfg& h) {
    const int64_t D = c.dim, ch = h.channels;
    switch (h.kind) {
        case VPE_HEAD_SEG: return (int64_t)h.classes * D + h.classes;
        case VPE_HEAD_DET: return 2 * (ch * D * 9 + ch) + (int64_t)h.classes * ch + h.classes + 4 * ch + 4;
        case VPE_HEAD_DEPTH: return 4 * (ch * D + ch) + 4 * (ch * ch * 9 + ch) + ch + 1;
        case VPE_HEAD_DPT: {
            const int64_t F = ch, oc0 = 3 * F / 4;
            int64_t n = 0;
            for (int i = 0; i < 4; ++i) n += (oc0 << i) * D + (oc0 << i);                   // tap projections
            n += oc0 * oc0 * 16 + oc0 + 4 * oc0 * oc0 * 4 + 2 * oc0 + 64 * oc0 * oc0 * 9 + 8 * oc0;   // up0, up1, down3
            for (int i = 0; i < 4; ++i) n += F * (oc0 << i) * 9;                            // l_i convolutions, no bias
            n += 14 * (F * F * 9 + F) + 4 * (F * F + F);                                    // 7 residual units, 4 output 1x1
            return n + (F / 2) * F * 9 + F / 2 + 32 * (F / 2) * 9 + 32 + 32 + 1;
        }
    }
    return -1;
}

// Multiply-accumulate work of one head run (x2 = FLOP), for balancing heads over streams.
double head_flops(const vpe_engine& e, const Head& h);

// Returns an empty string when the configuration is acceptable.
std::string validate(const vpe_backbone_cfg* c, const vpe_head_cfg* heads, int n_heads) {
    char buf[256];
    if (!c) return "backbone_cfg is null";
    if (n_heads < 0 || (n_heads > 0 && !heads)) return "heads is null";
    if (c->dim <= 0 || c->heads <= 0 || c->dim != c->heads * 64) return "dim must equal heads * 64";
    if (c->dim > 2048) return "dim above 2048 is not supported";
    if (c->depth < 1 || c->mlp_hidden < 64 || c->mlp_hidden % 64) return "depth >= 1 and mlp_hidden a multiple of 64 required";
    if (c->mlp_kind != VPE_MLP_GELU && c->mlp_kind != VPE_MLP_SWIGLU) return "unknown mlp_kind";
    if (c->dtype != VPE_F32 && c->dtype != VPE_BF16) return "unknown dtype";
    if (c->registers < 0 || c->registers > 64) return "registers out of range";
    if (c->batch < 1) return "batch must be >= 1";
    if (c->img_h < 14 || c->img_w < 14 || c->img_h % 14 || c->img_w % 14) return "img_h and img_w must be positive multiples of 14";
    if (c->ring_slots < 1 || c->ring_slots > 64) return "ring_slots must be in 1..64";
    if (!(c->ln_eps > 0.0f)) return "ln_eps must be positive";
    for (int k = 0; k < 4; ++k) {
        if (c->taps[k] < 1 || c->taps[k] > c->depth) return "taps must lie in 1..depth";
        if (k && c->taps[k] <= c->taps[k - 1]) return "taps must be strictly increasing";
    }
    if (c->taps[3] != c->depth) return "taps[3] must equal depth";
    if (!c->weights) return "backbone weights pointer is null";
    if ((int64_t)c->weights_bytes != 4 * backbone_floats(*c)) {
        snprintf(buf, sizeof buf, "backbone weights_bytes is %llu, expected %lld", (unsigned long long)c->weights_bytes,
                 (long long)(4 * backbone_floats(*c)));
        return buf;
    }
    for (int i = 0; i < n_heads; ++i) {
        const vpe_head_cfg& h = heads[i];
        if (h.kind != VPE_HEAD_SEG && h.kind != VPE_HEAD_DEPTH && h.kind != VPE_HEAD_DET && h.kind != VPE_HEAD_DPT)
            return "unknown head kind";
        if (h.kind == VPE_HEAD_DPT && h.channels > 256) return "a DPT head takes channels in 64..256";
        if (h.every_n < 1) return "every_n must be >= 1";
        if ((h.kind == VPE_HEAD_SEG || h.kind == VPE_HEAD_DET) && (h.classes < 1 || h.classes > 256)) return "classes must be in 1..256";
        if (h.kind != VPE_HEAD_SEG && (h.channels < 64 || h.channels % 64 || h.channels > 1024))
            return "channels must be a multiple of 64 in 64..1024";
        if (!h.weights) return "head weights pointer is null";
        if ((int64_t)h.weights_bytes != 4 * head_floats(*c, h)) {
            snprintf(buf, sizeof buf, "head %d weights_bytes is %llu, expected %lld", i,
                     (unsigned long long)h.weights_bytes, (long long)(4 * head_floats(*c, h)));
            return buf;
        }
    }
    return "";
}

void derive(vpe_engine& e, const vpe_backbone_cfg& c, const vpe_head_cfg* heads, int n_heads) {
    e.cfg = c;
    e.cfg.weights = nullptr;
    e.bf = c.dtype == VPE_BF16;
    e.esz = e.bf ? 2 : 4;
    e.host_only = false;
    e.graphs = (c.flags & VPE_FLAG_GRAPHS) != 0;
    e.timing = (c.flags & VPE_FLAG_TIMING) != 0;
    e.D = c.dim; e.L = c.depth; e.nh = c.heads; e.Mh = c.mlp_hidden;
    e.F = c.mlp_hidden * (c.mlp_kind == VPE_MLP_SWIGLU ? 2 : 1);
    e.R = c.registers; e.B = c.batch; e.H = c.img_h; e.W = c.img_w;
    e.gh = c.img_h / 14; e.gw = c.img_w / 14; e.P = e.gh * e.gw;
    e.N = 1 + e.R + e.P; e.T = e.B * e.N;
    e.npad = (int)rup(e.N, 64);
    e.S = c.ring_slots;
    e.lanes = std::max(1, std::min({c.encoder_lanes, c.ring_slots, MAX_LANES}));   // k encodes in flight need k slots
    e.heads.assign(n_heads, Head());
    for (int i = 0; i < n_heads; ++i) {
        e.heads[i].kind = heads[i].kind;
        e.heads[i].classes = heads[i].classes;
        e.heads[i].ch = heads[i].channels;
        e.heads[i].every_n = heads[i].every_n;
        if (heads[i].kind == VPE_HEAD_DPT) {
            Dpt& d = e.heads[i].dpt;
            d.F = heads[i].channels;
            d.hp = (int)rup(d.F / 2, 64);
            for (int k = 0; k < 4; ++k) {
                d.oc[k] = (3 * d.F / 4) << k;
                d.ocp[k] = (int)rup(d.oc[k], 64);
            }
            const int gh = c.img_h / 14, gw = c.img_w / 14;
            const int hh[4] = {4 * gh, 2 * gh, gh, (gh + 1) / 2}, ww[4] = {4 * gw, 2 * gw, gw, (gw + 1) / 2};
            for (int k = 0; k < 4; ++k) { d.hh[k] = hh[k]; d.ww[k] = ww[k]; }
            // resizes: after the fusion stage of level 3, 2, 1 to the next level's grid, after level 0 to twice
            // its grid, and the output map to the image
            const int rh[5] = {gh, 2 * gh, 4 * gh, 8 * gh, c.img_h}, rw[5] = {gw, 2 * gw, 4 * gw, 8 * gw, c.img_w};
            for (int k = 0; k < 5; ++k) { d.rh[k] = rh[k]; d.rw[k] = rw[k]; }
        }
    }
}

// Hands out every device region; with b.base == nullptr it only measures.
double head_flops(const vpe_engine& e, const Head& h) {
    const double P = (double)e.B * e.P;
    switch (h.kind) {
        case VPE_HEAD_SEG: return P * e.D * h.classes;
        case VPE_HEAD_DET: return P * (9.0 * e.D * 2 * h.ch + 2.0 * h.ch * (h.classes + 4));
        case VPE_HEAD_DPT: {
            const double F = h.ch;
            // residual units on the 1/4, 1, 4, 16 grids, the output convolutions on the 64x and 196x grids
            return P * (7.5 * e.D * F + 9.0 * F * F * (2 * 0.25 + 4 * 1 + 4 * 4 + 4 * 16) + 9.0 * F * F / 2 * 64 + 9.0 * 64 * 64 * 196);
        }
        default: return P * (4.0 * e.D * h.ch + 85.0 * 9 * h.ch * h.ch);   // four 3x3 stages on 1 + 4 + 16 + 64 grids
    }
}

// Hands out the intermediate buffers of a seg / det / DPT-lite head (see HeadScratch) from `b`.
void place_head_scratch(const vpe_engine& e, const Head& h, Bump& b, HeadScratch& sc) {
    const uint64_t esz = e.esz, ch = h.ch, BP = (uint64_t)e.B * e.P;
    if (h.kind == VPE_HEAD_DET) {
        sc.tower = b.take(BP * 2 * ch * esz);
    } else if (h.kind == VPE_HEAD_DEPTH) {
        for (int s = 0; s < 4; ++s) sc.p[s] = b.take(BP * ch * esz);
        sc.z = b.take(BP * 64 * ch * esz);
        sc.r = b.take(BP * 64 * ch * esz);
        sc.d8 = (float*)b.take(4 * (ch / 64) * BP * 64);
    }
}

void layout(vpe_engine& e, Bump& b) {
    const uint64_t esz = e.esz;
    const uint64_t D = e.D, T = e.T, P = e.P, B = e.B;
    auto wrows = [&](int n) { return (uint64_t)rup(n, NPAD); };
    auto f32 = [&](uint64_t n) { return (float*)b.take(4 * n); };
    e.patch_w = b.take(wrows(e.D) * KPATCH_PAD * esz);
    e.patch_b = f32(D);
    e.special = f32((1 + e.R) * D);
    e.pos = f32(P * D);
    e.blk.resize(e.L);
    for (auto& w : e.blk) {
        w.ln1_g = f32(D); w.ln1_b = f32(D);
        w.qkv_w = b.take(wrows(3 * e.D) * D * esz); w.qkv_b = f32(3 * D); w.qkv_s = f32(3 * D);
        w.proj_w = b.take(wrows(e.D) * D * esz); w.proj_b = f32(D);
        w.ls1 = f32(D);
        w.ln2_g = f32(D); w.ln2_b = f32(D);
        w.fc1_w = b.take(wrows(e.F) * D * esz); w.fc1_b = f32(e.F); w.fc1_s = f32(e.F);
        w.fc2_w = b.take(wrows(e.D) * e.Mh * esz); w.fc2_b = f32(D);
        w.ls2 = f32(D);
    }
    e.norm_g = f32(D); e.norm_b = f32(D);
    e.zeros = b.take(256);
    e.lev0 = f32(T);
    for (int l = 0; l < e.lanes; ++l) {
        vpe_engine::Lane& L = e.lane[l];
        L.apatch = b.take(B * P * KPATCH_PAD * esz);
        L.x = f32(T * D);
        L.stats = f32(T * (D / 64) * 2);
        L.lev[0] = f32(T); L.lev[1] = f32(T);
        L.u = b.take(T * D * esz);
        // + ATTN_PAD rows / elements that the attention loader may prefetch past the end (never used)
        L.qk = b.take((T + ATTN_PAD) * 2 * D * esz);
        L.vt = b.take((B * D * e.npad + ATTN_PAD) * esz);
        L.att = b.take(T * D * esz);
        L.hid = b.take(T * e.Mh * esz);
    }
    e.feat.resize((size_t)e.S * 4);
    for (auto& f : e.feat) f = b.take(T * D * esz);
    for (auto& h : e.heads) {
        const uint64_t ch = h.ch, BP = B * P;
        if (h.kind == VPE_HEAD_SEG) {
            h.w0 = b.take(wrows(h.classes) * D * esz); h.b0 = f32(h.classes);
            h.logits = f32(BP * h.classes);
            h.classmap = (uint8_t*)b.take(B * e.H * e.W);
        } else if (h.kind == VPE_HEAD_DET) {
            h.w0 = b.take(wrows(2 * h.ch) * 9 * D * esz); h.b0 = f32(2 * ch);
            h.w1 = b.take(wrows(h.classes + 4) * 2 * ch * esz); h.b1 = f32(h.classes + 4);
            place_head_scratch(e, h, b, h.sc);
            h.logits = f32(BP * (h.classes + 4));
            h.classmap = (uint8_t*)b.take(BP);
        } else if (h.kind == VPE_HEAD_DPT) {
            Dpt& d = h.dpt;
            const uint64_t F = d.F;
            auto conv = [&](ConvW& c, int n_out, uint64_t k, bool bias = true) {
                c.w = b.take(wrows(n_out) * k * esz);
                c.b = bias ? f32(rup(n_out, 64)) : nullptr;
            };
            d.up_w[0] = b.take(16 * wrows(d.oc[0]) * D * esz); d.up_b[0] = f32(16 * d.oc[0]);
            d.up_w[1] = b.take(4 * wrows(d.oc[1]) * D * esz); d.up_b[1] = f32(4 * d.oc[1]);
            conv(d.proj[0], d.oc[2], D); conv(d.proj[1], d.oc[3], D);
            conv(d.down3, d.oc[3], 9 * d.ocp[3]);
            for (int i = 0; i < 4; ++i) conv(d.rn[i], d.F, 9 * d.ocp[i], false);
            for (int k = 3; k >= 0; --k) {
                if (k < 3) { conv(d.fa1[k], d.F, 9 * F); conv(d.fa2[k], d.F, 9 * F); }
                conv(d.fb1[k], d.F, 9 * F); conv(d.fb2[k], d.F, 9 * F);
                conv(d.fout[k], d.F, F);
            }
            conv(d.head1, d.F / 2, 9 * F);
            conv(d.head2, 64, 9 * d.hp);
            d.head3_w = f32(64);
            uint64_t n[4];
            for (int i = 0; i < 4; ++i) n[i] = B * d.hh[i] * d.ww[i];
            const uint64_t n_out = B * d.rh[3] * d.rw[3], n_img = B * e.H * e.W;
            for (int i = 0; i < 4; ++i) d.R[i] = b.take(n[i] * d.ocp[i] * esz);
            d.P3 = b.take(BP * d.ocp[3] * esz);
            d.G3 = b.take(n[3] * 9 * d.ocp[3] * esz);
            for (int i = 0; i < 4; ++i) { d.L[i] = f32(n[i] * F); d.Lr[i] = b.take(n[i] * F * esz); }
            d.t = b.take(n[0] * F * esz); d.sr = b.take(n[0] * F * esz);
            d.y = b.take(n[0] * F * esz); d.c = b.take(n[0] * F * esz);
            d.s = f32(n[0] * F); d.path[0] = f32(n[0] * F); d.path[1] = f32(n[0] * F);
            d.path0 = b.take(n_out * F * esz);
            d.o1 = b.take(n_out * d.hp * esz);
            d.u = b.take(n_img * d.hp * esz);
            d.dpart = f32(n_img);
            h.depth = f32(n_img);
            for (int r = 0; r < 5; ++r) { d.ty[r] = b.take(8 * (uint64_t)d.rh[r]); d.tx[r] = b.take(8 * (uint64_t)d.rw[r]); }
        } else {
            for (int s = 0; s < 4; ++s) { h.proj_w[s] = b.take(wrows(h.ch) * D * esz); h.proj_b[s] = f32(ch); }
            for (int s = 0; s < 4; ++s) { h.fuse_w[s] = b.take(wrows(h.ch) * 9 * ch * esz); h.fuse_b[s] = f32(ch); }
            h.out_w = f32(ch);
            place_head_scratch(e, h, b, h.sc);
            h.depth = f32(B * e.H * e.W);
        }
    }
}

// Walks a host fp32 blob in its documented order and places each tensor on the device.
struct Uploader {
    vpe_engine* e;
    const float* host;
    int64_t n, pos = 0;
    float* staging;
    const float* take(int64_t k) { const float* p = host + pos; pos += k; return p; }
    int f32(float* dst, int64_t k) {
        HIPCHK(e, hipMemcpy(dst, take(k), 4 * k, hipMemcpyHostToDevice));
        return 0;
    }
    // tensor of `count` floats -> dst rows/cols via relayout_kernel (see rowops.h)
    int relayout(int64_t count, void* dst, int n_rows, int n_cols, int64_t rs, int64_t cs, int mode, int cin,
                 int swiglu_half, int64_t dst_ld, int row_off, int col_off, const float* kscale = nullptr) {
        return relayout_host(take(count), count, dst, n_rows, n_cols, rs, cs, mode, cin, swiglu_half, dst_ld, row_off,
                             col_off, kscale);
    }
    // the same from any host array (a tensor derived from the blob's)
    int relayout_host(const float* src, int64_t count, void* dst, int n_rows, int n_cols, int64_t rs, int64_t cs, int mode,
                      int cin, int swiglu_half, int64_t dst_ld, int row_off, int col_off, const float* kscale = nullptr) {
        HIPCHK(e, hipMemcpy(staging, src, 4 * count, hipMemcpyHostToDevice));
        HIPCHK(e, launch_relayout(e->bf, staging, dst, n_rows, n_cols, rs, cs, mode, cin, swiglu_half, dst_ld,
                                  row_off, col_off, kscale, nullptr));
        HIPCHK(e, hipStreamSynchronize(nullptr));
        return 0;
    }
    // 3x3 kernel [n_out][cin][3][3] -> [n_out][9 cpad], column tap * cpad + ci; bias (may be absent) -> b
    int conv3(const ConvW& c, int n_out, int cin, int cpad, bool bias = true) {
        if (relayout((int64_t)n_out * cin * 9, c.w, n_out, 9 * cin, 0, cpad, 1, cin, 0, 9 * (int64_t)cpad, 0, 0)) return 1;
        return bias ? f32(c.b, n_out) : 0;
    }
    // 1x1 kernel [n_out][cin] with bias
    int conv1(const ConvW& c, int n_out, int cin) {
        if (relayout((int64_t)n_out * cin, c.w, n_out, cin, cin, 1, 0, 0, 0, cin, 0, 0)) return 1;
        return f32(c.b, n_out);
    }
    // y = x W + b weights stored [in][out]  ->  [out][in]
    int linear(void* dst, int in, int out, int swiglu_half = 0, const float* kscale = nullptr) {
        return relayout((int64_t)in * out, dst, out, in, 1, out, 0, 0, swiglu_half, in, 0, 0, kscale);
    }
    // after linear(.., gain) and the upload of `bias` (device, physical order): column sums and folded bias,
    // from the fp32 weight still in `staging`
    int fold_ln(int in, int out, int swiglu_half, const float* gain, const float* beta, float* colsum, float* bias) {
        HIPCHK(e, launch_ln_fold(e->bf, staging, in, out, swiglu_half, gain, beta, colsum, bias, nullptr));
        HIPCHK(e, hipStreamSynchronize(nullptr));
        return 0;
    }
};

#define TRY(x) do { int rc__ = (x); if (rc__) return rc__; } while (0)

int upload_backbone(vpe_engine& e, const float* blob, float* staging) {
    Uploader up{&e, blob, backbone_floats(e.cfg), 0, staging};
    const int D = e.D;
    // patch kernel [D][588] -> [D][640] (zero padded columns)
    TRY(up.relayout((int64_t)D * KPATCH, e.patch_w, D, KPATCH, KPATCH, 1, 0, 0, 0, KPATCH_PAD, 0, 0));
    const float* patch_b = up.take(D);
    HIPCHK(&e, hipMemcpy(e.patch_b, patch_b, 4 * (size_t)D, hipMemcpyHostToDevice));
    // special rows: CLS + pos[0], then the registers; remaining pos rows belong to the patches
    const float* cls = up.take(D);
    const float* reg = up.take((int64_t)e.R * D);
    const float* pos = up.take((int64_t)(1 + e.P) * D);
    std::vector<float> sp((size_t)(1 + e.R) * D);
    for (int d = 0; d < D; ++d) sp[d] = cls[d] + pos[d];
    if (e.R) memcpy(sp.data() + D, reg, sizeof(float) * (size_t)e.R * D);
    HIPCHK(&e, hipMemcpy(e.special, sp.data(), sp.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(&e, hipMemcpy(e.pos, pos + D, (size_t)e.P * D * 4, hipMemcpyHostToDevice));
    {   // level of a fresh frame's rows: what is known of a row before its image arrives, averaged over the width
        std::vector<float> lev((size_t)e.T);
        for (int n = 0; n < e.N; ++n) {
            double acc = 0.0;
            if (n < 1 + e.R) for (int d = 0; d < D; ++d) acc += sp[(size_t)n * D + d];
            else for (int d = 0; d < D; ++d) acc += (double)patch_b[d] + pos[(size_t)(n - e.R) * D + d];
            for (int b = 0; b < e.B; ++b) lev[(size_t)b * e.N + n] = (float)(acc / D);
        }
        HIPCHK(&e, hipMemcpy(e.lev0, lev.data(), lev.size() * 4, hipMemcpyHostToDevice));
    }
    const bool sw = e.cfg.mlp_kind == VPE_MLP_SWIGLU;
    for (auto& w : e.blk) {
        TRY(up.f32(w.ln1_g, D)); TRY(up.f32(w.ln1_b, D));
        TRY(up.linear(w.qkv_w, D, 3 * D, 0, w.ln1_g)); TRY(up.f32(w.qkv_b, 3 * D));
        TRY(up.fold_ln(D, 3 * D, 0, w.ln1_g, w.ln1_b, w.qkv_s, w.qkv_b));
        TRY(up.linear(w.proj_w, D, D)); TRY(up.f32(w.proj_b, D));
        TRY(up.f32(w.ls1, D));
        TRY(up.f32(w.ln2_g, D)); TRY(up.f32(w.ln2_b, D));
        TRY(up.linear(w.fc1_w, D, e.F, sw ? e.Mh : 0, w.ln2_g));
        if (sw) {   // bias follows the same physical column order as the re-laid weight
            const float* b = up.take(e.F);
            std::vector<float> pb(e.F);
            for (int n = 0; n < e.F; ++n) {
                const int grp = n >> 6, j = n & 63;
                pb[n] = b[j < 32 ? 32 * grp + j : e.Mh + 32 * grp + j - 32];
            }
            HIPCHK(&e, hipMemcpy(w.fc1_b, pb.data(), 4 * (size_t)e.F, hipMemcpyHostToDevice));
        } else {
            TRY(up.f32(w.fc1_b, e.F));
        }
        TRY(up.fold_ln(D, e.F, sw ? e.Mh : 0, w.ln2_g, w.ln2_b, w.fc1_s, w.fc1_b));
        TRY(up.linear(w.fc2_w, e.Mh, D)); TRY(up.f32(w.fc2_b, D));
        TRY(up.f32(w.ls2, D));
    }
    TRY(up.f32(e.norm_g, D)); TRY(up.f32(e.norm_b, D));
    return up.pos == up.n ? 0 : e.fail(VPE_EINVAL, "backbone blob size mismatch");
}

int upload_head(vpe_engine& e, Head& h, const float* blob, int64_t n, float* staging) {
    Uploader up{&e, blob, n, 0, staging};
    const int D = e.D, ch = h.ch;
    if (h.kind == VPE_HEAD_SEG) {
        TRY(up.relayout((int64_t)h.classes * D, h.w0, h.classes, D, D, 1, 0, 0, 0, D, 0, 0));
        TRY(up.f32(h.b0, h.classes));
    } else if (h.kind == VPE_HEAD_DET) {
        // both towers as one [2 ch][9 D] implicit-GEMM weight (class tower first)
        TRY(up.relayout((int64_t)ch * D * 9, h.w0, ch, 9 * D, 0, 0, 1, D, 0, 9 * D, 0, 0));
        TRY(up.f32(h.b0, ch));
        TRY(up.relayout((int64_t)ch * D * 9, h.w0, ch, 9 * D, 0, 0, 1, D, 0, 9 * D, ch, 0));
        TRY(up.f32(h.b0 + ch, ch));
        // block-diagonal 1x1: class logits read tower columns [0, ch), box offsets [ch, 2 ch)
        TRY(up.relayout((int64_t)h.classes * ch, h.w1, h.classes, ch, ch, 1, 0, 0, 0, 2 * ch, 0, 0));
        TRY(up.f32(h.b1, h.classes));
        TRY(up.relayout((int64_t)4 * ch, h.w1, 4, ch, ch, 1, 0, 0, 0, 2 * ch, h.classes, ch));
        TRY(up.f32(h.b1 + h.classes, 4));
    } else if (h.kind == VPE_HEAD_DPT) {
        Dpt& d = h.dpt;
        const int F = d.F;
        const float *pw[2], *pb[2];
        for (int i = 0; i < 2; ++i) { pw[i] = up.take((int64_t)d.oc[i] * D); pb[i] = up.take(d.oc[i]); }
        TRY(up.conv1(d.proj[0], d.oc[2], D));
        TRY(up.conv1(d.proj[1], d.oc[3], D));
        // levels 0 and 1: out[(s y + dy, s x + dx)][co] = ub[co] + sum_ci uw[ci][co][dy][dx] (pb[ci] + sum_d pw[ci][d] x[d]):
        // one [oc][D] matrix and one bias vector per (dy, dx), composed here in double
        for (int i = 0; i < 2; ++i) {
            const int st = i == 0 ? 4 : 2, oc = d.oc[i];
            const float* uw = up.take((int64_t)oc * oc * st * st);
            const float* ub = up.take(oc);
            std::vector<double> acc((size_t)D);
            std::vector<float> wz((size_t)oc * D), bz((size_t)oc);
            const int64_t zstride = rup(oc, NPAD) * (int64_t)D * e.esz;
            for (int z = 0; z < st * st; ++z) {
                for (int co = 0; co < oc; ++co) {
                    std::fill(acc.begin(), acc.end(), 0.0);
                    double bb = ub[co];
                    for (int ci = 0; ci < oc; ++ci) {
                        const double u = uw[((int64_t)ci * oc + co) * st * st + z];
                        bb += u * pb[i][ci];
                        const float* row = pw[i] + (int64_t)ci * D;
                        for (int k = 0; k < D; ++k) acc[k] += u * row[k];
                    }
                    for (int k = 0; k < D; ++k) wz[(size_t)co * D + k] = (float)acc[k];
                    bz[co] = (float)bb;
                }
                TRY(up.relayout_host(wz.data(), (int64_t)oc * D, (char*)d.up_w[i] + z * zstride, oc, D, D, 1, 0, 0, 0, D, 0, 0));
                HIPCHK(&e, hipMemcpy(d.up_b[i] + (int64_t)z * oc, bz.data(), 4 * (size_t)oc, hipMemcpyHostToDevice));
            }
        }
        TRY(up.conv3(d.down3, d.oc[3], d.oc[3], d.ocp[3]));
        for (int i = 0; i < 4; ++i) TRY(up.conv3(d.rn[i], F, d.oc[i], d.ocp[i], false));
        for (int k = 3; k >= 0; --k) {
            if (k < 3) { TRY(up.conv3(d.fa1[k], F, F, F)); TRY(up.conv3(d.fa2[k], F, F, F)); }
            TRY(up.conv3(d.fb1[k], F, F, F)); TRY(up.conv3(d.fb2[k], F, F, F));
            TRY(up.conv1(d.fout[k], F, F));
        }
        TRY(up.conv3(d.head1, F / 2, F, F));
        TRY(up.conv3(d.head2, 32, F / 2, d.hp));
        TRY(up.f32(d.head3_w, 32));
        d.head3_b = *up.take(1);
        // aligned-corner taps: output index y of `out` samples sits at y (in - 1) / (out - 1)
        const int in_h[5] = {d.hh[3], d.hh[2], d.hh[1], d.hh[0], d.rh[3]}, in_w[5] = {d.ww[3], d.ww[2], d.ww[1], d.ww[0], d.rw[3]};
        for (int r = 0; r < 5; ++r)
            for (int axis = 0; axis < 2; ++axis) {
                const int in = axis ? in_w[r] : in_h[r], out = axis ? d.rw[r] : d.rh[r];
                std::vector<AcTap> tab((size_t)out);
                for (int y = 0; y < out; ++y) {
                    const int64_t num = (int64_t)y * (in - 1), den = out > 1 ? out - 1 : 1;
                    tab[y].i0 = (int)std::min<int64_t>(num / den, in - 1);
                    tab[y].w1 = (float)((double)(num % den) / (double)den);
                }
                HIPCHK(&e, hipMemcpy(axis ? d.tx[r] : d.ty[r], tab.data(), sizeof(AcTap) * tab.size(), hipMemcpyHostToDevice));
            }
    } else {
        for (int s = 0; s < 4; ++s) {
            TRY(up.relayout((int64_t)ch * D, h.proj_w[s], ch, D, D, 1, 0, 0, 0, D, 0, 0));
            TRY(up.f32(h.proj_b[s], ch));
        }
        for (int s = 0; s < 4; ++s) {
            TRY(up.relayout((int64_t)ch * ch * 9, h.fuse_w[s], ch, 9 * ch, 0, 0, 1, ch, 0, 9 * ch, 0, 0));
            TRY(up.f32(h.fuse_b[s], ch));
        }
        TRY(up.f32(h.out_w, ch));
        h.out_b = *up.take(1);
    }
    return up.pos == up.n ? 0 : e.fail(VPE_EINVAL, "head blob size mismatch");
}

GemmArgs plain_gemm(const void* A, int64_t lda, const void* W, const float* bias, int M, int N, int K) {
    GemmArgs a{};
    a.A = A; a.lda = lda; a.W = W; a.bias = bias; a.M = M; a.N = N; a.K = K;
    a.a_rpi = M > 0 ? M : 1; a.a_istride = 0; a.a_off = 0;
    a.o_rpi = M > 0 ? M : 1; a.o_istride = 0; a.o_off = 0;
    a.epi = EPI_STORE; a.act = ACT_NONE; a.out_f32 = 0;
    return a;
}

// ------------------------------------------------------------------ launch sequences
// A GEMM that consumes LayerNorm(x) of the lane's residual stream with the LayerNorm folded in: A is the copy
// of x in the engine dtype (x itself for fp32 engines), statistics come from the producers' epilogues.
// The 16-bit copy is stored relative to a per-row level: `level` is the one the current copy was written
// against, `next_level` receives the rows' means for the next copy (fp32 engines read x itself: no levels).
GemmArgs ln_gemm(const vpe_engine& e, const vpe_engine::Lane& L, const void* W, const float* bias, const float* colsum, int N,
                 const float* level, float* next_level) {
    GemmArgs a = plain_gemm(e.bf ? (const void*)L.u : (const void*)L.x, e.D, W, bias, e.T, N, e.D);
    a.ln_stats = L.stats; a.ln_colsum = colsum; a.ln_groups = e.D / 64; a.ln_eps = e.cfg.ln_eps;
    if (e.bf) { a.ln_level = level; a.ln_level_out = next_level; }
    return a;
}

// A GEMM whose epilogue updates the residual stream: also refreshes its copy (against `level`) and its row
// statistics.
void produce_stats(const vpe_engine& e, const vpe_engine::Lane& L, GemmArgs& a, const float* level) {
    a.out = L.x; a.ldo = e.D;
    a.st_out = L.stats;
    a.xb_out = e.bf ? L.u : nullptr;
    a.xb_level = e.bf ? level : nullptr;
}

int enqueue_encoder_body(vpe_engine& e, int slot, int lane, hipStream_t s) {
    const int D = e.D, T = e.T, dt = e.bf;
    const vpe_engine::Lane& L = e.lane[lane];
    {   // patch embedding: [B P][640] x [D][640]^T + bias + pos -> residual stream rows of the patches
        GemmArgs a = plain_gemm(L.apatch, KPATCH_PAD, e.patch_w, e.patch_b, e.B * e.P, D, KPATCH_PAD);
        a.epi = EPI_PATCH; a.pos = e.pos;
        a.o_rpi = e.P; a.o_istride = e.N; a.o_off = 1 + e.R;
        produce_stats(e, L, a, e.lev0);
        HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
    }
    // levels alternate between the lane's two buffers: each LayerNorm-consuming GEMM reads the level its input
    // was stored against and writes the rows' means into the other buffer, for the producer that follows it
    const float* level = e.lev0;
    int nxt = 0;
    int tap = 0;
    for (int l = 0; l < e.L; ++l) {
        const BlockW& w = e.blk[l];
        {
            GemmArgs a = ln_gemm(e, L, w.qkv_w, w.qkv_b, w.qkv_s, 3 * D, level, L.lev[nxt]);
            level = L.lev[nxt]; nxt ^= 1;
            a.epi = EPI_QKV; a.out = L.qk; a.ldo = 2 * D; a.out2 = L.vt; a.ntok = e.N; a.npad = e.npad; a.dim = D;
            HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
        }
        {
            AttnArgs a{L.qk, L.vt, L.att, e.B, e.N, e.npad, D, e.nh, 0.125f * 1.4426950408889634f, ATTN_PAD, e.lanes > 1};
            HIPCHK(&e, launch_attention(dt, a, s));
        }
        {
            GemmArgs a = plain_gemm(L.att, D, w.proj_w, w.proj_b, T, D, D);
            a.epi = EPI_RESID; a.gamma = w.ls1;
            produce_stats(e, L, a, level);
            HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
        }
        {
            GemmArgs a = ln_gemm(e, L, w.fc1_w, w.fc1_b, w.fc1_s, e.F, level, L.lev[nxt]);
            level = L.lev[nxt]; nxt ^= 1;
            a.out = L.hid; a.ldo = e.Mh;
            if (e.cfg.mlp_kind == VPE_MLP_SWIGLU) a.epi = EPI_SWIGLU;
            else a.act = ACT_GELU;
            HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
        }
        {
            GemmArgs a = plain_gemm(L.hid, e.Mh, w.fc2_w, w.fc2_b, T, D, e.Mh);
            a.epi = EPI_RESID; a.gamma = w.ls2;
            produce_stats(e, L, a, level);
            HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
        }
        if (tap < 4 && l + 1 == e.cfg.taps[tap]) {
            HIPCHK(&e, launch_layernorm(dt, L.x, T, D, e.norm_g, e.norm_b, e.cfg.ln_eps, e.feat[slot * 4 + tap], s));
            ++tap;
        }
    }
    return 0;
}

// 1x1 convolution on the patch rows of a feature map: skips CLS / register rows via the row map
GemmArgs tokens_gemm(vpe_engine& e, const void* feat, const void* W, const float* bias, int N) {
    GemmArgs a = plain_gemm(feat, e.D, W, bias, e.B * e.P, N, e.D);
    a.a_rpi = e.P; a.a_istride = e.N; a.a_off = 1 + e.R;
    return a;
}

GemmArgs conv3_gemm(vpe_engine& e, const void* in, int C, int B, int h, int w, int istride, int off,
                    const void* W, const float* bias, int N) {
    GemmArgs a = plain_gemm(in, C, W, bias, B * h * w, N, 9 * C);
    a.zeros = e.zeros;
    a.a_istride = istride; a.a_off = off; a.cH = h; a.cW = w; a.cC = C;
    a.act = ACT_RELU;
    return a;
}

// Full DPT head (see Dpt).  The residual trunk (l_i, the sums s_k, the paths) is kept in fp32 and added in the
// convolution epilogues; convolution operands are copies in the engine dtype, written through ReLU where the
// next convolution wants that.  The 1x1 output convolution of a fusion stage runs before the resize (on the
// smaller grid): both are linear and the resize weights sum to one, so the order only changes rounding.
int enqueue_dpt(vpe_engine& e, Head& h, int slot, hipStream_t s) {
    Dpt& d = h.dpt;
    const int dt = e.bf, F = d.F, B = e.B;
    void* const* f = &e.feat[slot * 4];
    auto conv = [&](const void* in, int cin_pad, int lvl_h, int lvl_w, const ConvW& w, int n_out, int act) {
        GemmArgs a = conv3_gemm(e, in, cin_pad, B, lvl_h, lvl_w, lvl_h * lvl_w, 0, w.w, w.b, n_out);
        a.act = act;
        return a;
    };
    // reassemble, levels 0 and 1: one batched launch each, problem z = (dy, dx) writes pixel (s y + dy, s x + dx)
    for (int i = 0; i < 2; ++i) {
        const int st = i == 0 ? 4 : 2, oc = d.oc[i], cp = d.ocp[i];
        GemmArgs a = tokens_gemm(e, f[i], d.up_w[i], d.up_b[i], oc);
        a.out = d.R[i]; a.ldo = (int64_t)st * cp;                  // consecutive grid columns are st pixels apart
        a.o_rpi = e.gw; a.o_istride = e.gw * st; a.o_off = 0;      // consecutive grid rows st pixel rows apart
        a.nz = st * st; a.z_a = 0; a.z_w = rup(oc, NPAD) * (int64_t)e.D * e.esz; a.z_bias = oc;
        a.z_inner = st; a.z_out = (int64_t)cp * e.esz; a.z_out2 = (int64_t)e.gw * st * cp * e.esz;
        HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
    }
    {   // level 2: the projection itself; level 3: projection, then 3x3 stride 2 as gather + GEMM
        GemmArgs a = tokens_gemm(e, f[2], d.proj[0].w, d.proj[0].b, d.oc[2]);
        a.out = d.R[2]; a.ldo = d.ocp[2];
        HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
        GemmArgs p3 = tokens_gemm(e, f[3], d.proj[1].w, d.proj[1].b, d.oc[3]);
        p3.out = d.P3; p3.ldo = d.ocp[3];
        HIPCHK(&e, launch_gemm(dt, p3, A_PLAIN, s));
        HIPCHK(&e, launch_gather3x3s2(dt, d.P3, B, e.gh, e.gw, d.ocp[3], d.G3, s));
        GemmArgs g = plain_gemm(d.G3, 9 * (int64_t)d.ocp[3], d.down3.w, d.down3.b, B * d.hh[3] * d.ww[3], d.oc[3], 9 * d.ocp[3]);
        g.out = d.R[3]; g.ldo = d.ocp[3];
        HIPCHK(&e, launch_gemm(dt, g, A_PLAIN, s));
    }
    for (int i = 0; i < 4; ++i) {   // l_i = 3x3 conv to F channels: fp32 trunk + ReLU copy
        GemmArgs a = conv(d.R[i], d.ocp[i], d.hh[i], d.ww[i], d.rn[i], F, ACT_NONE);
        a.out = d.L[i]; a.out_f32 = 1; a.ldo = F; a.twin = d.Lr[i]; a.twin_relu = 1;
        HIPCHK(&e, launch_gemm(dt, a, A_CONV3, s));
    }
    const float* path = nullptr;
    for (int k = 3; k >= 0; --k) {
        const int hk = d.hh[k], wk = d.ww[k], r = 3 - k;
        const float* trunk = d.L[k];
        const void* trunk_relu = d.Lr[k];
        if (k < 3) {   // s_k = path + unit_a(l_k)
            GemmArgs c1 = conv(d.Lr[k], F, hk, wk, d.fa1[k], F, ACT_RELU);
            c1.out = d.t; c1.ldo = F;
            HIPCHK(&e, launch_gemm(dt, c1, A_CONV3, s));
            GemmArgs c2 = conv(d.t, F, hk, wk, d.fa2[k], F, ACT_NONE);
            c2.out = d.s; c2.out_f32 = 1; c2.ldo = F; c2.add1 = d.L[k]; c2.add2 = path; c2.twin = d.sr; c2.twin_relu = 1;
            HIPCHK(&e, launch_gemm(dt, c2, A_CONV3, s));
            trunk = d.s;
            trunk_relu = d.sr;
        }
        GemmArgs c1 = conv(trunk_relu, F, hk, wk, d.fb1[k], F, ACT_RELU);
        c1.out = d.t; c1.ldo = F;
        HIPCHK(&e, launch_gemm(dt, c1, A_CONV3, s));
        GemmArgs c2 = conv(d.t, F, hk, wk, d.fb2[k], F, ACT_NONE);      // unit_b(s_k), only needed as an operand
        c2.out = d.y; c2.ldo = F; c2.add1 = trunk;
        HIPCHK(&e, launch_gemm(dt, c2, A_CONV3, s));
        GemmArgs o = plain_gemm(d.y, F, d.fout[k].w, d.fout[k].b, B * hk * wk, F, F);
        o.out = d.c; o.ldo = F;
        HIPCHK(&e, launch_gemm(dt, o, A_PLAIN, s));
        if (k > 0) {
            float* next = d.path[k & 1];
            HIPCHK(&e, launch_resize_ac(dt, 1, d.c, B, hk, wk, F, F, d.ty[r], d.tx[r], d.rh[r], d.rw[r], F, next, s));
            path = next;
        } else {
            HIPCHK(&e, launch_resize_ac(dt, 0, d.c, B, hk, wk, F, F, d.ty[r], d.tx[r], d.rh[r], d.rw[r], F, d.path0, s));
        }
    }
    GemmArgs h1 = conv(d.path0, F, d.rh[3], d.rw[3], d.head1, F / 2, ACT_NONE);
    h1.out = d.o1; h1.ldo = d.hp;
    HIPCHK(&e, launch_gemm(dt, h1, A_CONV3, s));
    HIPCHK(&e, launch_resize_ac(dt, 0, d.o1, B, d.rh[3], d.rw[3], d.hp, F / 2, d.ty[4], d.tx[4], e.H, e.W, d.hp, d.u, s));
    // last 3x3 (ReLU) with the 32 -> 1 projection taken in its epilogue; rows 32..63 of the weight are zero
    GemmArgs h2 = conv(d.u, d.hp, e.H, e.W, d.head2, 64, ACT_RELU);
    h2.epi = EPI_ROWDOT; h2.gamma = d.head3_w; h2.out = d.dpart; h2.ldo = 1;
    HIPCHK(&e, launch_gemm(dt, h2, A_CONV3, s));
    HIPCHK(&e, launch_rowsum_relu(d.dpart, 1, d.head3_b, (int64_t)B * e.H * e.W, h.depth, s));
    return 0;
}

int enqueue_head_body(vpe_engine& e, Head& h, const HeadScratch& sc, int slot, hipStream_t s) {
    const int dt = e.bf, BP = e.B * e.P;
    void* const* f = &e.feat[slot * 4];
    if (h.kind == VPE_HEAD_DPT) return enqueue_dpt(e, h, slot, s);
    if (h.kind == VPE_HEAD_SEG) {
        GemmArgs a = tokens_gemm(e, f[3], h.w0, h.b0, h.classes);
        a.out = h.logits; a.ldo = h.classes; a.out_f32 = 1;
        HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
        HIPCHK(&e, launch_seg_upsample_argmax(h.logits, e.B, e.gh, e.gw, h.classes, e.H, e.W, h.classmap, s));
    } else if (h.kind == VPE_HEAD_DET) {
        GemmArgs a = conv3_gemm(e, f[3], e.D, e.B, e.gh, e.gw, e.N, 1 + e.R, h.w0, h.b0, 2 * h.ch);
        a.out = sc.tower; a.ldo = 2 * h.ch;
        HIPCHK(&e, launch_gemm(dt, a, A_CONV3, s));
        GemmArgs o = plain_gemm(sc.tower, 2 * h.ch, h.w1, h.b1, BP, h.classes + 4, 2 * h.ch);
        o.out = h.logits; o.ldo = h.classes + 4; o.out_f32 = 1;
        HIPCHK(&e, launch_gemm(dt, o, A_PLAIN, s));
        HIPCHK(&e, launch_argmax_rows(h.logits, BP, h.classes, h.classes + 4, h.classmap, s));
    } else {
        // the four tap projections are independent problems of one shape: one batched launch when their
        // operands are evenly spaced in memory (they are, by construction of the workspace layout)
        const int64_t za = (const char*)f[2] - (const char*)f[3], zw = (const char*)h.proj_w[1] - (const char*)h.proj_w[0];
        const int64_t zo = (const char*)sc.p[1] - (const char*)sc.p[0], zb = h.proj_b[1] - h.proj_b[0];
        bool even = true;
        for (int st = 1; st < 4; ++st)
            even = even && (const char*)f[3 - st] - (const char*)f[3] == st * za &&
                   (const char*)h.proj_w[st] - (const char*)h.proj_w[0] == st * zw &&
                   (const char*)sc.p[st] - (const char*)sc.p[0] == st * zo && h.proj_b[st] - h.proj_b[0] == st * zb;
        for (int st = 0; st < (even ? 1 : 4); ++st) {
            GemmArgs a = tokens_gemm(e, f[3 - st], h.proj_w[st], h.proj_b[st], h.ch);
            a.out = sc.p[st]; a.ldo = h.ch;
            if (even) { a.nz = 4; a.z_a = za; a.z_w = zw; a.z_out = zo; a.z_bias = zb; }
            HIPCHK(&e, launch_gemm(dt, a, A_PLAIN, s));
        }
        for (int st = 0; st < 4; ++st) {
            const int hs = e.gh << st, wsz = e.gw << st;
            const void* in = sc.p[0];
            if (st) {
                HIPCHK(&e, launch_fuse_upsample(dt, sc.p[st], e.gh, e.gw, sc.r, e.B, hs, wsz, h.ch, sc.z, s));
                in = sc.z;
            }
            GemmArgs a = conv3_gemm(e, in, h.ch, e.B, hs, wsz, hs * wsz, 0, h.fuse_w[st], h.fuse_b[st], h.ch);
            if (st < 3) {
                a.out = sc.r; a.ldo = h.ch;
            } else {
                // last stage: the 1-channel projection is taken in the epilogue (per 64-channel group), the
                // 256-channel map itself is never written
                a.epi = EPI_ROWDOT; a.gamma = h.out_w; a.out = sc.d8; a.ldo = h.ch / 64;
            }
            HIPCHK(&e, launch_gemm(dt, a, A_CONV3, s));
        }
        HIPCHK(&e, launch_depth_output(sc.d8, h.ch / 64, h.out_b, e.B, 8 * e.gh, 8 * e.gw, e.H, e.W, h.depth, s));
    }
    return 0;
}

// Capture `body` into an executable graph.  The capture stream exists only for the duration of the capture:
// a standing extra stream would hold a share of a hardware queue next to the streams that do the work.
template <typename Fn>
int capture(vpe_engine& e, hipGraphExec_t* out, Fn body) {
    hipStream_t cs = nullptr;
    HIPCHK(&e, hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
    hipError_t eb = hipStreamBeginCapture(cs, hipStreamCaptureModeRelaxed);
    if (eb != hipSuccess) { (void)hipStreamDestroy(cs); HIPCHK(&e, eb); }
    const int rc = body(cs);
    hipGraph_t g = nullptr;
    const hipError_t ec = hipStreamEndCapture(cs, &g);
    (void)hipStreamDestroy(cs);
    if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
    HIPCHK(&e, ec);
    const hipError_t ei = hipGraphInstantiate(out, g, nullptr, nullptr, 0);
    (void)hipGraphDestroy(g);
    HIPCHK(&e, ei);
    return 0;
}

void destroy_engine(vpe_engine* e) {
    if (!e) return;
    if (!e->host_only) {
        (void)hipDeviceSynchronize();
        for (auto g : e->enc_graphs) if (g) (void)hipGraphExecDestroy(g);
        for (auto& h : e->heads) {
            for (auto g : h.graphs) if (g) (void)hipGraphExecDestroy(g);
        }
        for (auto hs : e->head_streams) if (hs) (void)hipStreamDestroy(hs);
        for (auto ev : e->ready) if (ev) (void)hipEventDestroy(ev);
        for (auto ev : e->done) if (ev) (void)hipEventDestroy(ev);
        for (auto& L : e->lane) {
            if (L.stream) (void)hipStreamDestroy(L.stream);
            for (hipEvent_t ev : {L.done, L.t_begin, L.t_end}) if (ev) (void)hipEventDestroy(ev);
        }
        for (auto& h : e->heads)
            for (hipEvent_t ev : {h.t_begin, h.t_end}) if (ev) (void)hipEventDestroy(ev);
        if (e->owns_ws && e->ws) (void)hipFree(e->ws);
    }
    delete e;
}

}  // namespace

// ====================================================================== C ABI
extern "C" {

int vpe_workspace_bytes(const vpe_backbone_cfg* cfg, const vpe_head_cfg* heads, int n_heads, uint64_t* bytes) {
    const std::string v = validate(cfg, heads, n_heads);
    if (!v.empty() || !bytes) { g_create_error = v.empty() ? "bytes is null" : v; return VPE_EINVAL; }
    vpe_engine e;
    derive(e, *cfg, heads, n_heads);
    Bump b;
    layout(e, b);
    *bytes = (uint64_t)rup((int64_t)b.off, 256);
    return VPE_OK;
}

int vpe_create(const vpe_backbone_cfg* cfg, const vpe_head_cfg* heads, int n_heads, void* workspace,
               uint64_t workspace_bytes, vpe_engine** out) {
    if (out) *out = nullptr;
    const std::string v = validate(cfg, heads, n_heads);
    if (!v.empty() || !out) { g_create_error = v.empty() ? "out is null" : v; return VPE_EINVAL; }
    vpe_engine* e = new vpe_engine();
    derive(*e, *cfg, heads, n_heads);
    e->host_only = (cfg->flags & VPE_FLAG_HOST_ONLY) != 0;
    e->wall_clock = (cfg->flags & VPE_FLAG_WALL_CLOCK) != 0;
    e->t0 = std::chrono::steady_clock::now();
    Bump measure;
    layout(*e, measure);
    const uint64_t need = (uint64_t)rup((int64_t)measure.off, 256);
    auto bail = [&](int code) { g_create_error = e->err; destroy_engine(e); return code; };
    const int nh = (int)e->heads.size();
    e->slot_frame.assign(e->S, -1);
    e->slot_time.assign(e->S, std::nan(""));
    e->done_set.assign((size_t)e->S * std::max(nh, 1), 0);
    if (e->host_only) { *out = e; return VPE_OK; }

    if (workspace) {
        if (workspace_bytes < need || ((uintptr_t)workspace & 255)) {
            e->fail(VPE_EINVAL, "workspace too small or not 256-byte aligned");
            return bail(VPE_EINVAL);
        }
        e->ws = (char*)workspace;
    } else {
        if (hipMalloc((void**)&e->ws, need) != hipSuccess) {
            e->fail(VPE_ENOMEM, "hipMalloc of the engine workspace failed (is a HIP device present?)");
            return bail(VPE_ENOMEM);
        }
        e->owns_ws = true;
    }
    e->ws_bytes = need;
    auto hip = [&](hipError_t rc, const char* what) {
        if (rc == hipSuccess) return 0;
        e->fail(VPE_EHIP, std::string(what) + ": " + hipGetErrorString(rc));
        return 1;
    };
    if (hip(hipGetDevice(&e->device), "hipGetDevice")) return bail(VPE_EHIP);
    if (hip(static_scratch(e->device, &e->static_ptr), "hipGetSymbolAddress(scratch)")) return bail(VPE_EHIP);
    if (hip(hipMemset(e->ws, 0, need), "hipMemset")) return bail(VPE_EHIP);
    if (hip(configure_attention(), "configure_attention")) return bail(VPE_EHIP);
    if (hip(configure_gemm(), "configure_gemm")) return bail(VPE_EHIP);
    if (hip(configure_gemm_bf16(), "configure_gemm_bf16")) return bail(VPE_EHIP);
    if (hip(configure_gemm_f32(), "configure_gemm_f32")) return bail(VPE_EHIP);
    Bump real;
    real.base = e->ws;
    layout(*e, real);

    // staging for one tensor at a time (freed before returning)
    int64_t big = (int64_t)e->D * std::max({3 * e->D, e->F, e->Mh, KPATCH});
    for (auto& h : e->heads) big = std::max<int64_t>(big, (int64_t)h.ch * 9 * std::max(e->D, h.ch));
    for (auto& h : e->heads) big = std::max<int64_t>(big, (int64_t)h.classes * e->D);
    for (auto& h : e->heads)
        if (h.kind == VPE_HEAD_DPT)
            big = std::max<int64_t>({big, (int64_t)h.dpt.oc[3] * h.dpt.oc[3] * 9, (int64_t)h.dpt.oc[3] * e->D});
    float* staging = nullptr;
    if (hip(hipMalloc((void**)&staging, 4 * big), "hipMalloc(staging)")) return bail(VPE_ENOMEM);
    int rc = upload_backbone(*e, (const float*)cfg->weights, staging);
    for (int i = 0; i < nh && !rc; ++i)
        rc = upload_head(*e, e->heads[i], (const float*)heads[i].weights, head_floats(*cfg, heads[i]), staging);
    (void)hipFree(staging);
    if (rc) return bail(rc);

    // Streams.  A process gets few hardware queues (four by default) and streams beyond that number share
    // them, which serialises work that was meant to overlap; so the engine keeps its concurrently active
    // streams within that budget: `lanes` encoder streams plus head streams, heads sharing a stream (heaviest
    // first onto the least loaded) when they outnumber what is left.
    for (int l = 0; l < e->lanes; ++l) {
        if (hip(hipStreamCreateWithFlags(&e->lane[l].stream, hipStreamNonBlocking), "hipStreamCreate")) return bail(VPE_EHIP);
        if (hip(hipEventCreateWithFlags(&e->lane[l].done, hipEventDisableTiming), "hipEventCreate")) return bail(VPE_EHIP);
    }
    if (nh > 0) {
        int ns = cfg->head_streams > 0 ? cfg->head_streams : std::max(1, HW_QUEUES - e->lanes);
        ns = std::min(ns, nh);
        e->head_streams.assign(ns, nullptr);
        for (auto& hs : e->head_streams)
            if (hip(hipStreamCreateWithFlags(&hs, hipStreamNonBlocking), "hipStreamCreate")) return bail(VPE_EHIP);
        std::vector<int> order(nh);
        for (int i = 0; i < nh; ++i) order[i] = i;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return head_flops(*e, e->heads[a]) > head_flops(*e, e->heads[b]); });
        std::vector<double> load(ns, 0.0);
        for (int i : order) {
            const int k = (int)(std::min_element(load.begin(), load.end()) - load.begin());
            e->heads[i].stream = e->head_streams[k];
            load[k] += head_flops(*e, e->heads[i]);
        }
    }
    e->ready.assign(e->S, nullptr);
    e->done.assign((size_t)e->S * std::max(nh, 1), nullptr);
    for (auto& ev : e->ready)
        if (hip(hipEventCreateWithFlags(&ev, hipEventDisableTiming), "hipEventCreate")) return bail(VPE_EHIP);
    for (auto& ev : e->done)
        if (hip(hipEventCreateWithFlags(&ev, hipEventDisableTiming), "hipEventCreate")) return bail(VPE_EHIP);
    if (e->timing) {
        for (int l = 0; l < e->lanes; ++l)
            for (hipEvent_t* ev : {&e->lane[l].t_begin, &e->lane[l].t_end})
                if (hip(hipEventCreate(ev), "hipEventCreate")) return bail(VPE_EHIP);
        for (auto& h : e->heads)
            for (hipEvent_t* ev : {&h.t_begin, &h.t_end})
                if (hip(hipEventCreate(ev), "hipEventCreate")) return bail(VPE_EHIP);
    }
    e->enc_graphs.assign((size_t)e->S * e->lanes, nullptr);
    for (auto& h : e->heads) h.graphs.assign(e->S, nullptr);
    if (hip(hipDeviceSynchronize(), "hipDeviceSynchronize")) return bail(VPE_EHIP);
    *out = e;
    return VPE_OK;
}

int vpe_preprocess_u8(const uint8_t* frames, int batch, int src_h, int src_w, float* images, int dst_h, int dst_w,
                      const float mean[3], const float std[3], void* stream) {
    if (!frames || !images || !mean || !std) { g_create_error = "null pointer"; return VPE_EINVAL; }
    if (batch < 1 || src_h < 1 || src_w < 1 || dst_h < 1 || dst_w < 1) { g_create_error = "sizes must be positive"; return VPE_EINVAL; }
    // 32-bit indices inside a frame
    if ((int64_t)src_h * src_w * 3 >= (int64_t(1) << 31) || (int64_t)dst_h * dst_w >= (int64_t(1) << 31)) { g_create_error = "frame too large"; return VPE_EINVAL; }
    for (int c = 0; c < 3; ++c)
        if (!(std[c] > 0.0f) || !std::isfinite(mean[c]) || !std::isfinite(std[c])) { g_create_error = "std must be positive and finite, mean finite"; return VPE_EINVAL; }
    const hipError_t rc = launch_preprocess_u8(frames, batch, src_h, src_w, dst_h, dst_w, mean, std, images, (hipStream_t)stream);
    if (rc != hipSuccess) { g_create_error = std::string("preprocess launch: ") + hipGetErrorString(rc); return VPE_EHIP; }
    return VPE_OK;
}

int vpe_next_encode_stream(vpe_engine* e, void** stream) {
    if (!e) return VPE_EINVAL;
    if (!stream) return e->fail(VPE_EINVAL, "stream is null");
    *stream = e->host_only ? nullptr : (void*)e->lane[e->frames % e->lanes].stream;
    return VPE_OK;
}

int vpe_encode(vpe_engine* e, const float* images, void* stream, vpe_feat* out) {
    return vpe_encode_at(e, images, stream, std::nan(""), out);
}

int vpe_encode_at(vpe_engine* e, const float* images, void* stream, double t_seconds, vpe_feat* out) {
    if (!e) return VPE_EINVAL;
    if (!out) return e->fail(VPE_EINVAL, "out is null");
    if (!images && !e->host_only) return e->fail(VPE_EINVAL, "images is null");
    if (std::isinf(t_seconds)) return e->fail(VPE_EINVAL, "frame time is not finite");
    if (std::isnan(t_seconds) && e->wall_clock)
        t_seconds = std::max(e->last_time, std::chrono::duration<double>(std::chrono::steady_clock::now() - e->t0).count());
    if (!std::isnan(t_seconds)) {
        if (e->have_time && t_seconds < e->last_time) return e->fail(VPE_EINVAL, "frame time went backwards");
        e->last_time = t_seconds;
        e->have_time = true;
    }
    const int64_t frame = e->frames;
    const int slot = (int)(frame % e->S);
    const int nh = (int)e->heads.size();
    if (!e->host_only) {
        const int ln = (int)(frame % e->lanes);
        vpe_engine::Lane& L = e->lane[ln];
        hipStream_t s = stream ? (hipStream_t)stream : L.stream;
        // the slot's previous frame may still be read by heads (or still be written): wait on the GPU
        for (int h = 0; h < nh; ++h)
            if (e->done_set[(size_t)slot * nh + h]) HIPCHK(e, hipStreamWaitEvent(s, e->done[(size_t)slot * nh + h], 0));
        if (e->slot_frame[slot] >= 0) HIPCHK(e, hipStreamWaitEvent(s, e->ready[slot], 0));
        // a lane's scratch is single-instance: order after the lane's previous encode
        if (L.used) HIPCHK(e, hipStreamWaitEvent(s, L.done, 0));
        if (e->timing) HIPCHK(e, hipEventRecord(L.t_begin, s));
        HIPCHK(e, launch_im2col(e->bf, images, e->B, e->H, e->W, KPATCH_PAD, L.apatch, e->special, 1 + e->R,
                                e->N, e->D, L.x, e->bf ? L.u : nullptr, L.stats, e->bf ? e->lev0 : nullptr, s));
        if (e->graphs) {
            hipGraphExec_t& ge = e->enc_graphs[(size_t)slot * e->lanes + ln];
            if (!ge) TRY(capture(*e, &ge, [&](hipStream_t cs) { return enqueue_encoder_body(*e, slot, ln, cs); }));
            HIPCHK(e, hipGraphLaunch(ge, s));
        } else {
            TRY(enqueue_encoder_body(*e, slot, ln, s));
        }
        if (e->timing) HIPCHK(e, hipEventRecord(L.t_end, s));
        HIPCHK(e, hipEventRecord(L.done, s));
        L.used = true;
        e->last_lane = ln;
        HIPCHK(e, hipEventRecord(e->ready[slot], s));
    }
    for (int h = 0; h < nh; ++h) e->done_set[(size_t)slot * nh + h] = 0;
    // the ring overwrites its oldest frame; heads that never asked about it (or a later one) are told
    if (e->slot_frame[slot] >= 0)
        for (Head& h : e->heads)
            if (h.seen < e->slot_frame[slot]) ++h.overflow;
    e->slot_frame[slot] = frame;
    e->slot_time[slot] = t_seconds;
    e->frames = frame + 1;
    out->slot = slot;
    out->reserved = 0;
    out->frame = frame;
    return VPE_OK;
}

namespace {
// The limit in Hz: may a frame stamped t run, and if so move the due time on.
bool hz_allows(Head& h, double t) {
    if (!(h.period > 0.0) || std::isnan(t)) return true;
    if (h.due_set && t < h.due - 1e-6 * h.period) return false;
    // accumulate while the head keeps up; after a gap of more than a period start again from this frame
    h.due = h.due_set && t - h.due < h.period ? h.due + h.period : t + h.period;
    h.due_set = true;
    return true;
}

// Enqueue one run of a head on the frame in `slot` (already checked to be current and due).
// `sc` = the intermediate buffers to use; `replay` = false launches the kernels one by one even on an engine with
// graphs (a replay is tied to the buffers it was captured with, and the first one instantiates a graph, which allocates).
int start_head(vpe_engine* e, int head, int slot, int64_t frame, void* stream, const HeadScratch& sc, bool replay) {
    Head& h = e->heads[head];
    const int nh = (int)e->heads.size();
    if (!e->host_only) {
        hipStream_t s = stream ? (hipStream_t)stream : h.stream;
        HIPCHK(e, hipStreamWaitEvent(s, e->ready[slot], 0));
        // the head's scratch and outputs are single-instance: order after its previous run
        if (h.ran) HIPCHK(e, hipStreamWaitEvent(s, h.last_done, 0));
        if (e->timing) HIPCHK(e, hipEventRecord(h.t_begin, s));
        if (e->graphs && replay) {
            if (!h.graphs[slot])
                TRY(capture(*e, &h.graphs[slot], [&](hipStream_t cs) { return enqueue_head_body(*e, h, h.sc, slot, cs); }));
            HIPCHK(e, hipGraphLaunch(h.graphs[slot], s));
        } else {
            TRY(enqueue_head_body(*e, h, sc, slot, s));
        }
        if (e->timing) HIPCHK(e, hipEventRecord(h.t_end, s));
        hipEvent_t ev = e->done[(size_t)slot * nh + head];
        HIPCHK(e, hipEventRecord(ev, s));
        h.last_done = ev;
    }
    e->done_set[(size_t)slot * nh + head] = 1;
    h.ran = true;
    h.last_run_frame = frame;
    ++h.runs;
    return VPE_OK;
}
}  // namespace

int vpe_run_head(vpe_engine* e, int head, vpe_feat fh, void* stream) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size()) return e->fail(VPE_EINVAL, "unknown head");
    if (fh.slot < 0 || fh.slot >= e->S || fh.frame < 0 || fh.frame >= e->frames || fh.frame % e->S != fh.slot)
        return e->fail(VPE_EINVAL, "feature handle was not produced by this engine");
    Head& h = e->heads[head];
    h.seen = std::max(h.seen, fh.frame);
    if (fh.frame % h.every_n != 0) { ++h.skips; return VPE_SKIPPED; }
    if (e->slot_frame[fh.slot] != fh.frame) return e->fail(VPE_ESTALE, "slot has been reused by a later frame");
    if (!hz_allows(h, e->slot_time[fh.slot])) { ++h.skips; return VPE_SKIPPED; }
    return start_head(e, head, fh.slot, fh.frame, stream, h.sc, true);
}

int vpe_run_head_static(vpe_engine* e, int head, vpe_feat fh, void* stream) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size()) return e->fail(VPE_EINVAL, "unknown head");
    if (fh.slot < 0 || fh.slot >= e->S || fh.frame < 0 || fh.frame >= e->frames || fh.frame % e->S != fh.slot)
        return e->fail(VPE_EINVAL, "feature handle was not produced by this engine");
    Head& h = e->heads[head];
    if (h.kind == VPE_HEAD_DPT) return e->fail(VPE_EINVAL, "vpe_run_head_static: the full DPT head is not supported (its padded maps rely on a cleared workspace)");
    // carve the head's intermediate buffers out of the static array (same order and alignment as in a workspace)
    Bump b;
    b.base = (char*)e->static_ptr;     // null for host-only engines: then this only measures
    HeadScratch sc;
    place_head_scratch(*e, h, b, sc);
    if (b.off > STATIC_SCRATCH_BYTES) {
        char buf[192];
        snprintf(buf, sizeof buf, "vpe_run_head_static: this head needs %llu bytes of scratch, the static array holds %llu",
                 (unsigned long long)b.off, (unsigned long long)STATIC_SCRATCH_BYTES);
        return e->fail(VPE_EINVAL, buf);
    }
    if (!e->host_only) {
        int dev = -1;
        HIPCHK(e, hipGetDevice(&dev));
        if (dev != e->device) return e->fail(VPE_EINVAL, "vpe_run_head_static: the engine's GPU is not the current device");
    }
    h.seen = std::max(h.seen, fh.frame);
    if (fh.frame % h.every_n != 0) { ++h.skips; return VPE_SKIPPED; }
    if (e->slot_frame[fh.slot] != fh.frame) return e->fail(VPE_ESTALE, "slot has been reused by a later frame");
    if (!hz_allows(h, e->slot_time[fh.slot])) { ++h.skips; return VPE_SKIPPED; }
    return start_head(e, head, fh.slot, fh.frame, stream, sc, false);
}

int vpe_run_head_latest(vpe_engine* e, int head, void* stream, vpe_feat* ran_on) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size()) return e->fail(VPE_EINVAL, "unknown head");
    Head& h = e->heads[head];
    if (e->frames - 1 <= h.seen) return VPE_SKIPPED;                 // nothing new since the head last asked
    if (!e->host_only && h.ran) {
        const hipError_t q = hipEventQuery(h.last_done);
        if (q == hipErrorNotReady) { ++h.busy; return VPE_BUSY; }
        HIPCHK(e, q);
    }
    // newest frame that is still in the ring and whose features are complete on the device
    int64_t newest = -1;
    for (int64_t f = e->frames - 1; f > h.seen && f >= e->frames - e->S; --f) {
        if (!e->host_only) {
            const hipError_t q = hipEventQuery(e->ready[f % e->S]);
            if (q == hipErrorNotReady) continue;
            HIPCHK(e, q);
        }
        newest = f;
        break;
    }
    if (newest < 0) return VPE_SKIPPED;                              // the new frames are still being encoded
    const int64_t skipped_over = newest - 1 - h.seen;                // frames between the last one asked about and this one
    h.seen = newest;
    h.missed += skipped_over;
    const int slot = (int)(newest % e->S);
    if (h.last_run_frame >= 0 && newest - h.last_run_frame < h.every_n) { ++h.skips; return VPE_SKIPPED; }
    if (!hz_allows(h, e->slot_time[slot])) { ++h.skips; return VPE_SKIPPED; }
    const int rc = start_head(e, head, slot, newest, stream, h.sc, true);
    if (rc == VPE_OK && ran_on) { ran_on->slot = slot; ran_on->reserved = 0; ran_on->frame = newest; }
    return rc;
}

int vpe_frame_ready(vpe_engine* e, vpe_feat fh) {
    if (!e) return VPE_EINVAL;
    if (fh.slot < 0 || fh.slot >= e->S || fh.frame < 0 || fh.frame >= e->frames || fh.frame % e->S != fh.slot)
        return e->fail(VPE_EINVAL, "feature handle was not produced by this engine");
    if (e->slot_frame[fh.slot] != fh.frame) return VPE_ESTALE;
    if (e->host_only) return VPE_OK;
    const hipError_t q = hipEventQuery(e->ready[fh.slot]);
    if (q == hipErrorNotReady) return VPE_BUSY;
    HIPCHK(e, q);
    return VPE_OK;
}

int vpe_head_counters(vpe_engine* e, int head, int64_t out[8]) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size() || !out) return e->fail(VPE_EINVAL, "unknown head or null output");
    const Head& h = e->heads[head];
    out[0] = h.runs; out[1] = h.skips; out[2] = h.missed; out[3] = h.overflow;
    out[4] = h.busy; out[5] = h.last_run_frame; out[6] = h.seen; out[7] = 0;
    return VPE_OK;
}

int vpe_set_head_rate(vpe_engine* e, int head, int every_n_frames) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size()) return e->fail(VPE_EINVAL, "unknown head");
    if (every_n_frames < 1) return e->fail(VPE_EINVAL, "every_n_frames must be >= 1");
    e->heads[head].every_n = every_n_frames;
    return VPE_OK;
}

int vpe_set_head_rate_hz(vpe_engine* e, int head, double max_hz) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size()) return e->fail(VPE_EINVAL, "unknown head");
    if (!(max_hz >= 0.0) || std::isinf(max_hz)) return e->fail(VPE_EINVAL, "max_hz must be finite and >= 0");
    Head& h = e->heads[head];
    h.period = max_hz > 0.0 ? 1.0 / max_hz : 0.0;
    h.due_set = false;
    return VPE_OK;
}

int vpe_feat_view(vpe_engine* e, vpe_feat fh, int tap, const void** dev_ptr, int64_t shape[3]) {
    if (!e) return VPE_EINVAL;
    if (tap < 0 || tap > 3 || !dev_ptr || !shape) return e->fail(VPE_EINVAL, "bad tap or null output");
    if (fh.slot < 0 || fh.slot >= e->S || fh.frame < 0 || fh.frame >= e->frames || fh.frame % e->S != fh.slot)
        return e->fail(VPE_EINVAL, "feature handle was not produced by this engine");
    if (e->slot_frame[fh.slot] != fh.frame) return e->fail(VPE_ESTALE, "slot has been reused by a later frame");
    *dev_ptr = e->host_only ? nullptr : e->feat[(size_t)fh.slot * 4 + tap];
    shape[0] = e->B; shape[1] = e->N; shape[2] = e->D;
    return VPE_OK;
}

int vpe_head_output(vpe_engine* e, int head, int which, const void** dev_ptr, int64_t shape[4]) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size() || !dev_ptr || !shape) return e->fail(VPE_EINVAL, "unknown head or null output");
    const Head& h = e->heads[head];
    shape[0] = e->B; shape[1] = shape[2] = shape[3] = 1;
    if (h.kind == VPE_HEAD_SEG && which == 0) { *dev_ptr = h.logits; shape[1] = e->gh; shape[2] = e->gw; shape[3] = h.classes; }
    else if (h.kind == VPE_HEAD_SEG && which == 1) { *dev_ptr = h.classmap; shape[1] = e->H; shape[2] = e->W; }
    else if (h.kind == VPE_HEAD_DET && which == 0) { *dev_ptr = h.logits; shape[1] = e->gh; shape[2] = e->gw; shape[3] = h.classes + 4; }
    else if (h.kind == VPE_HEAD_DET && which == 1) { *dev_ptr = h.classmap; shape[1] = e->gh; shape[2] = e->gw; }
    else if ((h.kind == VPE_HEAD_DEPTH || h.kind == VPE_HEAD_DPT) && which == 0) { *dev_ptr = h.depth; shape[1] = e->H; shape[2] = e->W; }
    else return e->fail(VPE_EINVAL, "this head has no such output");
    return VPE_OK;
}

int vpe_sync(vpe_engine* e) {
    if (!e) return VPE_EINVAL;
    if (e->host_only) return VPE_OK;
    // every enqueue through the engine ends in an event of its own, whichever stream it went to: wait for those,
    // not for the device (other work of the process is none of the engine's business)
    for (int l = 0; l < e->lanes; ++l)
        if (e->lane[l].used) HIPCHK(e, hipEventSynchronize(e->lane[l].done));
    // (the slots' ready events follow the lanes' on the same streams; waiting for them too makes
    // vpe_frame_ready answer VPE_OK for every frame as soon as this returns)
    for (int sl = 0; sl < e->S; ++sl)
        if (e->slot_frame[sl] >= 0) HIPCHK(e, hipEventSynchronize(e->ready[sl]));
    for (Head& h : e->heads)
        if (h.ran) HIPCHK(e, hipEventSynchronize(h.last_done));
    return VPE_OK;
}

int vpe_head_done(vpe_engine* e, int head) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size()) return e->fail(VPE_EINVAL, "unknown head");
    const Head& h = e->heads[head];
    if (e->host_only || !h.ran) return VPE_OK;
    const hipError_t q = hipEventQuery(h.last_done);
    if (q == hipErrorNotReady) return VPE_BUSY;
    HIPCHK(e, q);
    return VPE_OK;
}

int vpe_wait_head(vpe_engine* e, int head) {
    if (!e) return VPE_EINVAL;
    if (head < 0 || head >= (int)e->heads.size()) return e->fail(VPE_EINVAL, "unknown head");
    const Head& h = e->heads[head];
    if (e->host_only || !h.ran) return VPE_OK;
    HIPCHK(e, hipEventSynchronize(h.last_done));
    return VPE_OK;
}

int vpe_stage_times(vpe_engine* e, float* encode_ms, float* head_ms, int n) {
    if (!e) return VPE_EINVAL;
    if (!e->timing) return e->fail(VPE_EINVAL, "the engine was not created with VPE_FLAG_TIMING");
    auto span = [&](bool ran, hipEvent_t b, hipEvent_t t, float* out) -> int {
        *out = -1.0f;
        if (!ran || e->host_only) return VPE_OK;
        const hipError_t q = hipEventQuery(t);
        if (q == hipErrorNotReady) return VPE_OK;              // still executing: no figure yet
        HIPCHK(e, q);
        HIPCHK(e, hipEventElapsedTime(out, b, t));
        return VPE_OK;
    };
    if (encode_ms) {
        const bool ran = e->last_lane >= 0;
        const vpe_engine::Lane& L = e->lane[ran ? e->last_lane : 0];
        TRY(span(ran, L.t_begin, L.t_end, encode_ms));
    }
    for (int i = 0; head_ms && i < n && i < (int)e->heads.size(); ++i)
        TRY(span(e->heads[i].ran, e->heads[i].t_begin, e->heads[i].t_end, head_ms + i));
    return VPE_OK;
}

int vpe_stats(vpe_engine* e, int64_t* frames, int64_t* head_runs, int64_t* head_skips, int n) {
    if (!e) return VPE_EINVAL;
    if (frames) *frames = e->frames;
    for (int i = 0; i < n && i < (int)e->heads.size(); ++i) {
        if (head_runs) head_runs[i] = e->heads[i].runs;
        if (head_skips) head_skips[i] = e->heads[i].skips;
    }
    return VPE_OK;
}

int vpe_time_kernel(vpe_engine* e, int which, int reps, float* ms_per_launch, double* flops, double* bytes) {
    if (!e) return VPE_EINVAL;
    if (e->host_only || reps < 1 || !ms_per_launch) return e->fail(VPE_EINVAL, "bad arguments");
    // the launches below write scratch of encoder lane 0 and of the depth head: nothing of the engine may be in flight
    TRY(vpe_sync(e));
    hipStream_t s = e->lane[0].stream;
    const vpe_engine::Lane& L0 = e->lane[0];
    hipEvent_t t0, t1;
    HIPCHK(e, hipEventCreate(&t0));
    HIPCHK(e, hipEventCreate(&t1));
    const int D = e->D, T = e->T, dt = e->bf;
    double fl = 0.0, by = 0.0;
    int launches = reps, rc = 0;
    Head* dh = nullptr;
    for (auto& h : e->heads) if (h.kind == VPE_HEAD_DEPTH) dh = &h;
    auto body = [&](bool timed) -> int {
        if (timed) HIPCHK(e, hipEventRecord(t0, s));
        for (int i = 0; i < (timed ? reps : 1); ++i) {
            if (which == 0) {
                GemmArgs a = ln_gemm(*e, L0, e->blk[0].qkv_w, e->blk[0].qkv_b, e->blk[0].qkv_s, 3 * D, L0.lev[1], nullptr);
                a.epi = EPI_QKV; a.out = L0.qk; a.ldo = 2 * D; a.out2 = L0.vt; a.ntok = e->N; a.npad = e->npad; a.dim = D;
                HIPCHK(e, launch_gemm(dt, a, A_PLAIN, s));
            } else if (which == 1) {
                AttnArgs a{L0.qk, L0.vt, L0.att, e->B, e->N, e->npad, D, e->nh, 0.125f * 1.4426950408889634f, ATTN_PAD, e->lanes > 1};
                HIPCHK(e, launch_attention(dt, a, s));
            } else if (which == 5 || which == 7) {
                // out-projection / fc2 of block 0 with the LayerScale residual epilogue (the residual stream of lane 0
                // accumulates over the repetitions; the next encode rewrites it)
                const BlockW& w = e->blk[0];
                GemmArgs a = which == 5 ? plain_gemm(L0.att, D, w.proj_w, w.proj_b, T, D, D)
                                        : plain_gemm(L0.hid, e->Mh, w.fc2_w, w.fc2_b, T, D, e->Mh);
                a.epi = EPI_RESID; a.gamma = which == 5 ? w.ls1 : w.ls2;
                produce_stats(*e, L0, a, L0.lev[1]);
                HIPCHK(e, launch_gemm(dt, a, A_PLAIN, s));
            } else if (which == 6 || which == 9) {
                GemmArgs a = ln_gemm(*e, L0, e->blk[0].fc1_w, e->blk[0].fc1_b, e->blk[0].fc1_s, e->F, L0.lev[1], nullptr);
                a.out = L0.hid; a.ldo = e->Mh;
                if (which == 9) { a.N = e->Mh; }             // plain store of the first mlp_hidden columns: no activation
                else if (e->cfg.mlp_kind == VPE_MLP_SWIGLU) a.epi = EPI_SWIGLU;
                else a.act = ACT_GELU;
                HIPCHK(e, launch_gemm(dt, a, A_PLAIN, s));
            } else if (which == 8) {
                HIPCHK(e, launch_activation(dt, L0.hid, T, e->Mh, e->cfg.mlp_kind == VPE_MLP_SWIGLU, s));
            } else if (which == 2) {
                // into the attention-output scratch: same size as a feature map, rewritten by the next encode before it is read
                HIPCHK(e, launch_layernorm(dt, L0.x, T, D, e->norm_g, e->norm_b, e->cfg.ln_eps, L0.att, s));
            } else if (which == 4) {
                // the stage input of that convolution: upsample of the tap projection + x2 upsample of the previous
                // stage's output, 8x the patch grid (bandwidth-bound: reads 1/4 of what it writes)
                HIPCHK(e, launch_fuse_upsample(dt, dh->sc.p[3], e->gh, e->gw, dh->sc.r, e->B, e->gh << 3, e->gw << 3, dh->ch, dh->sc.z, s));
            } else {
                // the largest 3x3 convolution of the depth head (last fusion stage, 8x the patch grid), same
                // shape, weights and buffers as in a head run; its timing does not depend on the values in z
                const int hs = e->gh << 3, wsz = e->gw << 3;
                GemmArgs a = conv3_gemm(*e, dh->sc.z, dh->ch, e->B, hs, wsz, hs * wsz, 0, dh->fuse_w[3], dh->fuse_b[3], dh->ch);
                a.epi = EPI_ROWDOT; a.gamma = dh->out_w; a.out = dh->sc.d8; a.ldo = dh->ch / 64;
                HIPCHK(e, launch_gemm(dt, a, A_CONV3, s));
            }
        }
        if (timed) HIPCHK(e, hipEventRecord(t1, s));
        return 0;
    };
    if (which < 0 || which > 9 || ((which == 3 || which == 4) && !dh)) rc = e->fail(VPE_EINVAL, "no such kernel to time");
    if (!rc) rc = body(false);   // warm-up launch
    if (!rc) rc = body(true);
    if (!rc && hipEventSynchronize(t1) != hipSuccess) rc = e->fail(VPE_EHIP, "hipEventSynchronize failed");
    float ms = 0.0f;
    if (!rc && hipEventElapsedTime(&ms, t0, t1) != hipSuccess) rc = e->fail(VPE_EHIP, "hipEventElapsedTime failed");
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (rc) return rc;
    const double esz = e->esz;
    if (which == 0) { fl = 2.0 * T * D * 3.0 * D; by = esz * ((double)T * D + 3.0 * D * D + 3.0 * T * D); }
    else if (which == 1) { fl = 4.0 * e->B * (double)e->N * e->N * D; by = esz * 4.0 * T * D; }
    else if (which == 2) { fl = 8.0 * T * D; by = (4.0 + esz) * T * D; }
    else if (which == 5) { fl = 2.0 * T * D * D; by = esz * ((double)T * D + (double)D * D) + (8.0 + esz) * T * D; }
    else if (which == 6) { fl = 2.0 * T * D * (double)e->F; by = esz * ((double)T * D + (double)D * e->F + (double)T * e->Mh); }
    else if (which == 8) {
        const double n = (double)T * e->Mh * (e->cfg.mlp_kind == VPE_MLP_SWIGLU ? 0.5 : 1.0);
        fl = 12.0 * n; by = esz * (e->cfg.mlp_kind == VPE_MLP_SWIGLU ? 3.0 : 2.0) * n;
    }
    else if (which == 9) { fl = 2.0 * T * D * (double)e->Mh; by = esz * ((double)T * D + (double)D * e->Mh + (double)T * e->Mh); }
    else if (which == 7) { fl = 2.0 * T * D * (double)e->Mh; by = esz * ((double)T * e->Mh + (double)D * e->Mh) + (8.0 + esz) * T * D; }
    else if (which == 4) {
        const double ch = dh->ch, pix = (double)e->B * e->P;
        fl = 14.0 * 64.0 * pix * ch;                                   // two bilinear blends and an add per output value
        by = esz * ch * pix * (1.0 + 16.0 + 64.0);                     // tap projection + previous stage in, stage input out
    }
    else {
        const double ch = dh->ch, pix = (double)e->B * e->P * 64.0;
        fl = 2.0 * 9.0 * ch * ch * pix;
        by = esz * (pix * ch + 9.0 * ch * ch) + 4.0 * pix;     // input map + weights in, one projected value per pixel out
    }
    *ms_per_launch = ms / launches;
    if (flops) *flops = fl;
    if (bytes) *bytes = by;
    return VPE_OK;
}

const char* vpe_last_error(vpe_engine* e) { return e ? e->err.c_str() : g_create_error.c_str(); }

void vpe_destroy(vpe_engine* e) { destroy_engine(e); }

}  // extern "C"
