// ckpt_pack_image: the pack step on its own. A list of tensors is gathered into the image of its
// checkpoint data region in device memory, without a context: no ring, no threads, no file.
// ckpt_pack_image_noalloc: the same for callers that cannot allocate; its tile table lives in a static
// device array of this file.
#include "engine_internal.hpp"
#include "tile_batch.hpp"

// The tile table of ckpt_pack_image_noalloc: room for kScratchTiles tiles (4 MiB), held by every GPU the
// library runs on until the process ends. In host code this name is only a stand-in for the symbol: the
// array's address on a device comes from hipGetSymbolAddress (scratch_on_current_device below) and only
// that address is ever handed to a kernel.
constexpr uint64_t kScratchTiles = 131072;
static __device__ __align__(256) unsigned char scratch[kScratchTiles * sizeof(ckpt_tile)];

namespace dsllm {
hipError_t launch_build_tiles(const TileBatch &bt, ckpt_tile *dev_table, hipStream_t stream);
}

using namespace dsllm;

namespace {

// What both entry points check before anything is launched: every tensor is device memory of the
// current GPU and lies inside its allocation, the destination is device memory of the same GPU, 16-byte
// aligned and large enough. Returns the data-region size and the number of tiles.
int check_pack_arguments(const ckpt_tensor_desc *tensors, size_t n, const void *dev_dst, uint64_t dst_bytes, uint64_t *data_bytes_out,
                         uint64_t *n_tiles_out) {
    if (!tensors || n == 0 || !dev_dst) return fail(CKPT_EINVAL, "null argument or empty tensor list");
    int dev = 0;
    HIP_TRY(nullptr, hipGetDevice(&dev));
    // 0: fine; 1: not device memory of this GPU; 2: runs past its allocation (queries only, nothing is allocated;
    // texts are put together on the failing path alone)
    auto on_this_gpu = [&](const void *p, uint64_t nbytes) -> int {
        hipPointerAttribute_t attr;
        hipError_t e = hipPointerGetAttributes(&attr, p);
        if (e != hipSuccess || attr.type != hipMemoryTypeDevice || attr.device != dev) { (void)hipGetLastError(); return 1; }
        void *base = nullptr; size_t span = 0;
        e = hipMemGetAddressRange(reinterpret_cast<hipDeviceptr_t *>(&base), &span, reinterpret_cast<hipDeviceptr_t>(const_cast<void *>(p)));
        if (e == hipSuccess && uint64_t(p) + nbytes > uint64_t(base) + span) return 2;
        if (e != hipSuccess) (void)hipGetLastError();
        return 0;
    };
    static const char *const why[] = {"", ": not device memory of the current GPU", ": range runs past its allocation"};
    uint64_t off = 0, tiles = 0;
    for (size_t k = 0; k < n; k++) {
        const ckpt_tensor_desc &d = tensors[k];
        if (d.dtype & CKPT_PLACE_HOST) return fail(CKPT_EINVAL, "tensor " + std::to_string(k) + ": host-resident objects cannot be packed on the device");
        if (!d.dev_ptr || d.nbytes == 0) return fail(CKPT_EINVAL, "tensor " + std::to_string(k) + ": null pointer or zero bytes");
        if (int bad = on_this_gpu(d.dev_ptr, d.nbytes)) return fail(CKPT_EINVAL, "tensor " + std::to_string(k) + why[bad]);
        tiles += tiles_of(off, d.nbytes, kTileBytes);
        off += (d.nbytes + kAlign - 1) / kAlign * kAlign;
    }
    if (uint64_t(dev_dst) % 16 != 0) return fail(CKPT_EINVAL, "destination must be 16-byte aligned");
    if (dst_bytes < off) return fail(CKPT_EINVAL, "destination smaller than the data region (" + std::to_string(off) + " bytes)");
    if (int bad = on_this_gpu(dev_dst, off)) return fail(CKPT_EINVAL, std::string("destination") + why[bad]);
    if (tiles > 0xFFFFFFFFull) return fail(CKPT_EINVAL, "more than 2^32 tiles");
    *data_bytes_out = off;
    *n_tiles_out = tiles;
    return CKPT_OK;
}

// Enqueues, on `stream`, the kernels that write the tile table into `dev_table` (room for n_tiles entries)
// and then the pack kernel over it. Allocates nothing, on either side.
int enqueue_pack_image(const ckpt_tensor_desc *tensors, size_t n, void *dev_dst, ckpt_tile *dev_table, uint64_t n_tiles,
                       hipStream_t stream) {
    TileBatch bt;
    bt.count = 0;
    uint64_t off = 0, tile = 0;
    for (size_t k = 0; k < n; k++) {
        const uint32_t j = bt.count++;
        bt.src[j] = uint64_t(tensors[k].dev_ptr);
        bt.data_off[j] = off;
        bt.nbytes[j] = tensors[k].nbytes;
        bt.first_tile[j] = uint32_t(tile);
        tile += tiles_of(off, tensors[k].nbytes, kTileBytes);
        off += (tensors[k].nbytes + kAlign - 1) / kAlign * kAlign;
        bt.first_tile[j + 1] = uint32_t(tile);
        if (bt.count == uint32_t(kTileBatch) || k + 1 == n) {
            HIP_TRY(nullptr, launch_build_tiles(bt, dev_table, stream));
            bt.count = 0;
        }
    }
    if (tile != n_tiles) return fail(CKPT_EINVAL, "internal: tile count changed between check and launch");
    HIP_TRY(nullptr, launch_pack(dev_table, n_tiles, dev_dst, 0, stream));
    return CKPT_OK;
}

// Where each device keeps its copy of `scratch` (every GPU has its own, at its own address): looked up once
// per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];

int scratch_on_current_device(void **out) {
    int dev = 0;
    HIP_TRY(nullptr, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CKPT_EINVAL, "device ordinal beyond what the scratch table foresees");
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(CKPT_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CKPT_OK;
}

}  // namespace

// Called by ckpt_init for its device, so that a caller who has a context never meets the first-use lookup
// (which may load the code object) inside a region where nothing may be allocated.
int dsllm::pack_scratch_setup() {
    void *p = nullptr;
    return scratch_on_current_device(&p);
}

extern "C" {

int ckpt_pack_image_noalloc(const ckpt_tensor_desc *tensors, size_t n, void *dev_dst, uint64_t dst_bytes, void *hip_stream) {
    uint64_t data_bytes = 0, n_tiles = 0;
    int r = check_pack_arguments(tensors, n, dev_dst, dst_bytes, &data_bytes, &n_tiles);
    if (r) return r;
    if (n_tiles > kScratchTiles)
        return fail(CKPT_EINVAL, "tensor list needs " + std::to_string(n_tiles) + " tiles, the static table holds " + std::to_string(kScratchTiles) +
                                     " (about 4 GiB of data region): use ckpt_pack_image");
    void *table = nullptr;
    r = scratch_on_current_device(&table);
    if (r) return r;
    // every entry the pack kernel reads is written by the table kernels just before it, on the same stream:
    // nothing of the previous call's table has to be cleared
    return enqueue_pack_image(tensors, n, dev_dst, static_cast<ckpt_tile *>(table), n_tiles, static_cast<hipStream_t>(hip_stream));
}

int ckpt_pack_image(const ckpt_tensor_desc *tensors, size_t n, void *dev_dst, uint64_t dst_bytes, void *hip_stream) {
    uint64_t data_bytes = 0, n_tiles = 0;
    int r = check_pack_arguments(tensors, n, dev_dst, dst_bytes, &data_bytes, &n_tiles);
    if (r) return r;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ckpt_tile *table = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&table), n_tiles * sizeof(ckpt_tile));
    if (e != hipSuccess) return fail(CKPT_ENOMEM, std::string("hipMalloc(tile table): ") + hipGetErrorString(e));
    r = enqueue_pack_image(tensors, n, dev_dst, table, n_tiles, stream);
    hipError_t es = hipStreamSynchronize(stream);   // the table must outlive the kernels that read it
    (void)hipFree(table);
    if (r) return r;
    if (es != hipSuccess) return fail(CKPT_EHIP, std::string("hipStreamSynchronize: ") + hipGetErrorString(es));
    return CKPT_OK;
}

}  // extern "C"
