// Host emulation of the pack and scatter kernels under AddressSanitizer (see hip/hip_runtime.h here).
// Builds random fragment layouts (all 16 start misalignments, ragged sizes, tiny and multi-tile
// tensors), plans them with the library's own planner, runs the real kernel source thread by thread,
// and checks (a) no access leaves the 16-byte-aligned hull of a tensor or the staging slot (ASan),
// (b) staging equals the expected packed image, (c) scatter restores the bytes and leaves every byte
// outside the tensors untouched.
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "../../paper_2406_10707_amd/csrc/pack_kernels.hip"
#include "../../paper_2406_10707_amd/csrc/plan.hpp"

thread_local dim3 threadIdx, blockIdx, blockDim, gridDim;
ssize_t emu_pwrite(int, const void *, size_t, off_t) { return -1; }   // no file is written here

static uint64_t rng_state;
static uint64_t rnd() {
    rng_state += 0x9E3779B97F4A7C15ull;
    uint64_t z = rng_state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct Hull { uint8_t *base; uint64_t hull_bytes; uint64_t lead; uint64_t nbytes; };   // tensor = base+lead .. +nbytes

int main(int argc, char **argv) {
    uint64_t seed = argc > 1 ? strtoull(argv[1], 0, 10) : 1;
    int n_tensors = argc > 2 ? atoi(argv[2]) : 200;
    rng_state = seed;
    using namespace dsllm;
    ckpt_config cfg{};
    cfg.dma_chunk_bytes = 64 << 10;
    cfg.pack_superchunk_bytes = 256 << 10;
    ResolvedConfig rc;
    std::string err;
    if (resolve_config(&cfg, &rc, &err)) { printf("config: %s\n", err.c_str()); return 2; }

    std::vector<Hull> hulls;
    std::vector<ckpt_tensor_desc> descs;
    std::vector<std::string> names;
    std::vector<int64_t> shapes(n_tensors);
    names.reserve(n_tensors);
    for (int k = 0; k < n_tensors; k++) {
        uint64_t lead = k < 16 ? k : rnd() % 16;                   // every misalignment at least once
        uint64_t nb;
        switch (rnd() % 6) {
            case 0: nb = 1 + rnd() % 40; break;                      // smaller than two words
            case 1: nb = 4096 - 16 + rnd() % 33; break;              // around one alignment unit
            case 2: nb = 32768 * (1 + rnd() % 2) - 32 + rnd() % 65; break;   // around one or two tiles
            case 3: nb = 65536 * (1 + rnd() % 3) + rnd() % 5000; break;
            case 4: nb = 16 * (1 + rnd() % 600); break;              // whole words
            default: nb = 1 + rnd() % 200000; break;
        }
        Hull h;
        h.lead = lead; h.nbytes = nb;
        h.hull_bytes = (lead + nb + 15) / 16 * 16;
        h.base = static_cast<uint8_t *>(aligned_alloc(16, h.hull_bytes));   // ASan guards both ends of the hull
        for (uint64_t i = 0; i < h.hull_bytes; i++) h.base[i] = uint8_t(rnd());
        hulls.push_back(h);
        names.push_back("t" + std::to_string(k));
        shapes[k] = int64_t(nb);
        ckpt_tensor_desc d{};
        d.name = names.back().c_str(); d.dtype = CKPT_U8; d.ndim = 1; d.shape = &shapes[k];
        d.dev_ptr = h.base + lead; d.nbytes = nb;
        descs.push_back(d);
    }
    Plan p;
    if (build_plan(descs.data(), descs.size(), rc, &p, &err)) { printf("plan: %s\n", err.c_str()); return 2; }
    const uint64_t SC = rc.pack_superchunk_bytes;

    // the tile table as the device builds it (batches of descriptors in the kernel arguments) must be the planner's
    {
        std::vector<ckpt_tile> table(p.tiles.size());
        TileBatch bt;
        bt.count = 0;
        uint64_t off = 0, tile = 0;
        for (size_t k = 0; k < descs.size(); k++) {
            const uint32_t j = bt.count++;
            bt.src[j] = uint64_t(descs[k].dev_ptr); bt.data_off[j] = off; bt.nbytes[j] = descs[k].nbytes; bt.first_tile[j] = uint32_t(tile);
            tile += tiles_of(off, descs[k].nbytes, kTileBytes);
            off += (descs[k].nbytes + 4095) / 4096 * 4096;
            bt.first_tile[j + 1] = uint32_t(tile);
            if (tile > table.size()) { printf("tiles_of counts %llu tiles, the planner %zu\n", (unsigned long long)tile, table.size()); return 1; }
            if (bt.count == uint32_t(kTileBatch) || k + 1 == descs.size()) { launch_build_tiles(bt, table.data(), nullptr); bt.count = 0; }
        }
        if (tile != p.tiles.size() || off != p.data_bytes) { printf("tile count or data size differs from the planner's\n"); return 1; }
        for (size_t i = 0; i < table.size(); i++) {
            const ckpt_tile &a = table[i], &b = p.tiles[i];
            if (a.src != b.src || a.dst_off != b.dst_off || a.copy_bytes != b.copy_bytes || a.total_bytes != b.total_bytes || a.reserved != 0) {
                printf("device-built tile %zu differs from the planner's\n", i);
                return 1;
            }
        }
    }

    // expected packed image
    std::vector<uint8_t> want(p.data_bytes, 0);
    for (size_t k = 0; k < hulls.size(); k++) memcpy(&want[p.tensors[k].file_off - p.header_bytes], hulls[k].base + hulls[k].lead, hulls[k].nbytes);

    // pack super-chunk by super-chunk into an exactly sized slot
    {
    std::vector<uint8_t> image(p.data_bytes);
    for (uint64_t sc = 0; sc < p.n_superchunks; sc++) {
        uint64_t bytes = p.superchunk_bytes(sc);
        uint8_t *slot = static_cast<uint8_t *>(aligned_alloc(16, bytes));
        memset(slot, 0xCC, bytes);
        uint64_t t0 = p.sc_first_tile[sc], t1 = p.sc_first_tile[sc + 1];
        launch_pack(p.tiles.data() + t0, t1 - t0, slot, sc * SC, nullptr, nullptr, nullptr);
        memcpy(&image[sc * SC], slot, bytes);
        free(slot);
    }
    if (image != want) {
        for (uint64_t i = 0; i < p.data_bytes; i++) if (image[i] != want[i]) { printf("pack mismatch at data offset %llu\n", (unsigned long long)i); break; }
        return 1;
    }
    }

    // scatter back into poisoned hulls
    std::vector<std::vector<uint8_t>> orig;
    for (auto &h : hulls) { orig.emplace_back(h.base, h.base + h.hull_bytes); memset(h.base, 0xA5, h.hull_bytes); }
    for (uint64_t sc = 0; sc < p.n_superchunks; sc++) {
        uint64_t bytes = p.superchunk_bytes(sc);
        uint8_t *slot = static_cast<uint8_t *>(aligned_alloc(16, bytes));
        memcpy(slot, &want[sc * SC], bytes);
        uint64_t t0 = p.sc_first_tile[sc], t1 = p.sc_first_tile[sc + 1];
        launch_scatter(p.tiles.data() + t0, t1 - t0, slot, sc * SC, nullptr);
        free(slot);
    }
    for (size_t k = 0; k < hulls.size(); k++) {
        auto &h = hulls[k];
        for (uint64_t i = 0; i < h.hull_bytes; i++) {
            bool inside = i >= h.lead && i < h.lead + h.nbytes;
            uint8_t expect = inside ? orig[k][i] : 0xA5;
            if (h.base[i] != expect) { printf("scatter mismatch tensor %zu byte %llu (lead %llu, nbytes %llu)\n", k, (unsigned long long)i, (unsigned long long)h.lead, (unsigned long long)h.nbytes); return 1; }
        }
        free(h.base);
    }
    printf("ok seed %llu tensors %d tiles %zu superchunks %llu data %llu\n", (unsigned long long)seed, n_tensors, p.tiles.size(), (unsigned long long)p.n_superchunks, (unsigned long long)p.data_bytes);
    return 0;
}
