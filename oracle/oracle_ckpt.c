/*
 * CPU oracle for the checkpoint snapshot path. TEST INFRASTRUCTURE ONLY: it may be called from
 * tests/, the smoke check and the benchmark's cpu_baseline leg, never from the product path.
 *
 * What it computes (paper: design principles "lazy non-blocking copies" and the three-phase save
 * of the Implementation section): the checkpoint of iteration i is the serialization of the exact
 * bytes every registered tensor holds after update i. The asynchronous machinery changes when
 * bytes move, never which bytes, so the oracle is the plain synchronous serializer: the caller
 * reads every tensor back with blocking copies at the iteration boundary and hands the host byte
 * arrays in; the oracle computes the header (file offset per tensor) and writes header, then each
 * tensor followed by zero padding, with sequential write() calls. The file layout is the one in
 * docs/FORMAT.md, implemented here from that page alone.
 *
 * One thread, no chunking, no overlap, no ring. Shares no code with the HIP library.
 */
#define _GNU_SOURCE
#include <errno.h>
#include <fcntl.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <sys/stat.h>
#include <unistd.h>

#define ORACLE_ALIGN 4096ull
#define ORACLE_FIXED 64ull

enum { ORACLE_OK = 0, ORACLE_BAD_ARG = 1, ORACLE_IO = 2, ORACLE_BAD_FILE = 3, ORACLE_MISMATCH = 4, ORACLE_NOMEM = 5 };

typedef struct {
    const char *name;      /* UTF-8, NUL terminated here; stored without the NUL */
    int32_t dtype;         /* 1 bf16, 2 f32, 3 f16, 4 u8, 5 i32, 6 i64 */
    uint32_t ndim;         /* 0..8 */
    const int64_t *shape;  /* ndim entries */
    void *host_bytes;      /* nbytes bytes on the host; may be NULL for header-only calls */
    uint64_t nbytes;
} oracle_tensor;

static const uint8_t MAGIC[8] = { 'D', 'S', 'L', 'L', 'M', 'C', 'K', 0x01 };

static uint64_t round_up(uint64_t x) { return (x + ORACLE_ALIGN - 1) / ORACLE_ALIGN * ORACLE_ALIGN; }

static uint64_t elsize(int32_t dtype)
{
    switch (dtype) {
    case 1: return 2; case 2: return 4; case 3: return 2; case 4: return 1; case 5: return 4; case 6: return 8;
    default: return 0;
    }
}

static void put_le(uint8_t *p, uint64_t v, int nbytes) { for (int i = 0; i < nbytes; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static uint64_t get_le(const uint8_t *p, int nbytes) { uint64_t v = 0; for (int i = 0; i < nbytes; i++) v |= (uint64_t)p[i] << (8 * i); return v; }

static int tensor_ok(const oracle_tensor *t)
{
    if (!t->name) return 0;
    size_t len = strlen(t->name);
    if (len < 1 || len > 65535) return 0;
    uint64_t es = elsize(t->dtype);
    if (es == 0 || t->ndim > 8) return 0;
    uint64_t numel = 1;
    for (uint32_t d = 0; d < t->ndim; d++) { if (t->shape[d] < 0) return 0; numel *= (uint64_t)t->shape[d]; }
    return t->nbytes > 0 && t->nbytes == es * numel;
}

static uint64_t entry_len(const oracle_tensor *t) { return 2 + strlen(t->name) + 1 + 1 + 8ull * t->ndim + 8 + 8; }

/* header_bytes for a tensor list: the fixed part plus all entries, rounded up to the alignment unit. */
uint64_t oracle_header_bytes(const oracle_tensor *ts, size_t n)
{
    uint64_t used = ORACLE_FIXED;
    for (size_t k = 0; k < n; k++) used += entry_len(&ts[k]);
    return round_up(used);
}

uint64_t oracle_data_bytes(const oracle_tensor *ts, size_t n)
{
    uint64_t total = 0;
    for (size_t k = 0; k < n; k++) total += round_up(ts[k].nbytes);
    return total;
}

/* File offset of tensor k: tensors follow the header in registration order, each starting on an
 * alignment boundary (FORMAT.md, data region). */
uint64_t oracle_tensor_offset(const oracle_tensor *ts, size_t n, size_t k)
{
    uint64_t off = oracle_header_bytes(ts, n);
    for (size_t j = 0; j < k; j++) off += round_up(ts[j].nbytes);
    return off;
}

/* Write the whole header (fixed part, table, zero fill) into out[0 .. header_bytes). */
int oracle_build_header(const oracle_tensor *ts, size_t n, uint64_t iter, uint8_t *out, uint64_t cap)
{
    for (size_t k = 0; k < n; k++) if (!tensor_ok(&ts[k])) return ORACLE_BAD_ARG;
    uint64_t hb = oracle_header_bytes(ts, n), db = oracle_data_bytes(ts, n);
    if (cap < hb) return ORACLE_BAD_ARG;
    memset(out, 0, hb);
    memcpy(out, MAGIC, 8);
    put_le(out + 8, 1, 4);
    put_le(out + 12, ORACLE_ALIGN, 4);
    put_le(out + 16, iter, 8);
    put_le(out + 24, n, 8);
    put_le(out + 32, hb, 8);
    put_le(out + 40, db, 8);
    put_le(out + 48, hb + db, 8);
    put_le(out + 56, 0, 8);
    uint8_t *p = out + ORACLE_FIXED;
    uint64_t off = hb;
    for (size_t k = 0; k < n; k++) {
        size_t len = strlen(ts[k].name);
        put_le(p, len, 2); p += 2;
        memcpy(p, ts[k].name, len); p += len;
        *p++ = (uint8_t)ts[k].dtype;
        *p++ = (uint8_t)ts[k].ndim;
        for (uint32_t d = 0; d < ts[k].ndim; d++) { put_le(p, (uint64_t)ts[k].shape[d], 8); p += 8; }
        put_le(p, off, 8); p += 8;
        put_le(p, ts[k].nbytes, 8); p += 8;
        off += round_up(ts[k].nbytes);
    }
    return ORACLE_OK;
}

static int write_all(int fd, const void *buf, uint64_t len)
{
    const uint8_t *p = (const uint8_t *)buf;
    while (len > 0) {
        size_t want = len > (1ull << 30) ? (size_t)(1ull << 30) : (size_t)len;
        ssize_t w = write(fd, p, want);
        if (w < 0) { if (errno == EINTR) continue; return ORACLE_IO; }
        p += w; len -= (uint64_t)w;
    }
    return ORACLE_OK;
}

static int read_all(int fd, void *buf, uint64_t len)
{
    uint8_t *p = (uint8_t *)buf;
    while (len > 0) {
        size_t want = len > (1ull << 30) ? (size_t)(1ull << 30) : (size_t)len;
        ssize_t r = read(fd, p, want);
        if (r < 0) { if (errno == EINTR) continue; return ORACLE_IO; }
        if (r == 0) return ORACLE_BAD_FILE;
        p += r; len -= (uint64_t)r;
    }
    return ORACLE_OK;
}

/* The serializer: header, then tensor after tensor with its zero padding, sequential write(). */
int oracle_serialize_file(const oracle_tensor *ts, size_t n, uint64_t iter, const char *path)
{
    uint64_t hb = oracle_header_bytes(ts, n);
    uint8_t *hdr = (uint8_t *)malloc(hb);
    if (!hdr) return ORACLE_NOMEM;
    int rc = oracle_build_header(ts, n, iter, hdr, hb);
    if (rc) { free(hdr); return rc; }
    for (size_t k = 0; k < n; k++) if (!ts[k].host_bytes) { free(hdr); return ORACLE_BAD_ARG; }
    int fd = open(path, O_WRONLY | O_CREAT | O_TRUNC, 0644);
    if (fd < 0) { free(hdr); return ORACLE_IO; }
    static const uint8_t zeros[ORACLE_ALIGN] = { 0 };
    rc = write_all(fd, hdr, hb);
    for (size_t k = 0; k < n && rc == ORACLE_OK; k++) {
        rc = write_all(fd, ts[k].host_bytes, ts[k].nbytes);
        if (rc == ORACLE_OK) rc = write_all(fd, zeros, round_up(ts[k].nbytes) - ts[k].nbytes);
    }
    if (close(fd) != 0 && rc == ORACLE_OK) rc = ORACLE_IO;
    free(hdr);
    return rc;
}

/* Same bytes into memory (for small cases). Returns file_bytes through *written. */
int oracle_serialize_mem(const oracle_tensor *ts, size_t n, uint64_t iter, uint8_t *out, uint64_t cap, uint64_t *written)
{
    uint64_t hb = oracle_header_bytes(ts, n), db = oracle_data_bytes(ts, n);
    if (cap < hb + db) return ORACLE_BAD_ARG;
    int rc = oracle_build_header(ts, n, iter, out, cap);
    if (rc) return rc;
    uint8_t *p = out + hb;
    for (size_t k = 0; k < n; k++) {
        if (!ts[k].host_bytes) return ORACLE_BAD_ARG;
        uint64_t padded = round_up(ts[k].nbytes);
        memcpy(p, ts[k].host_bytes, ts[k].nbytes);
        memset(p + ts[k].nbytes, 0, padded - ts[k].nbytes);
        p += padded;
    }
    if (written) *written = hb + db;
    return ORACLE_OK;
}

/* Streaming comparison of an existing file against what the oracle would write, without holding a
 * second copy of the data: returns ORACLE_MISMATCH and the first differing file offset. */
int oracle_compare_file(const oracle_tensor *ts, size_t n, uint64_t iter, const char *path, uint64_t *first_diff)
{
    uint64_t hb = oracle_header_bytes(ts, n), db = oracle_data_bytes(ts, n);
    if (first_diff) *first_diff = UINT64_MAX;
    uint8_t *hdr = (uint8_t *)malloc(hb);
    if (!hdr) return ORACLE_NOMEM;
    int rc = oracle_build_header(ts, n, iter, hdr, hb);
    if (rc) { free(hdr); return rc; }
    int fd = open(path, O_RDONLY);
    if (fd < 0) { free(hdr); return ORACLE_IO; }
    struct stat st;
    if (fstat(fd, &st) != 0) { close(fd); free(hdr); return ORACLE_IO; }
    if ((uint64_t)st.st_size != hb + db) { close(fd); free(hdr); if (first_diff) *first_diff = (uint64_t)st.st_size < hb + db ? (uint64_t)st.st_size : hb + db; return ORACLE_MISMATCH; }
    const uint64_t BUF = 8ull << 20;
    uint8_t *buf = (uint8_t *)malloc(BUF);
    if (!buf) { close(fd); free(hdr); return ORACLE_NOMEM; }
    uint64_t pos = 0;
    /* header */
    for (uint64_t done = 0; done < hb && rc == ORACLE_OK; ) {
        uint64_t m = hb - done < BUF ? hb - done : BUF;
        rc = read_all(fd, buf, m);
        if (rc == ORACLE_OK) for (uint64_t i = 0; i < m; i++) if (buf[i] != hdr[done + i]) { if (first_diff) *first_diff = pos + i; rc = ORACLE_MISMATCH; break; }
        done += m; pos += m;
    }
    for (size_t k = 0; k < n && rc == ORACLE_OK; k++) {
        const uint8_t *src = (const uint8_t *)ts[k].host_bytes;
        uint64_t padded = round_up(ts[k].nbytes);
        for (uint64_t done = 0; done < padded && rc == ORACLE_OK; ) {
            uint64_t m = padded - done < BUF ? padded - done : BUF;
            rc = read_all(fd, buf, m);
            if (rc == ORACLE_OK) for (uint64_t i = 0; i < m; i++) {
                uint8_t want = done + i < ts[k].nbytes ? src[done + i] : 0;
                if (buf[i] != want) { if (first_diff) *first_diff = pos + i; rc = ORACLE_MISMATCH; break; }
            }
            done += m; pos += m;
        }
    }
    free(buf); free(hdr); close(fd);
    return rc;
}

/* The same comparison for a run of tensors [first, first + count) only, so that a shard too large to be
 * held on the host a second time can be checked piece by piece: host_bytes is needed for those tensors
 * alone. Each piece also checks the file's size, and the piece that starts at tensor 0 the whole header.
 * A tensor's piece of the file is its nbytes bytes at the oracle's offset followed by zero bytes up to
 * the next alignment boundary. Pieces that together cover every tensor cover every byte of the file. */
int oracle_compare_file_span(const oracle_tensor *ts, size_t n, uint64_t iter, size_t first, size_t count, const char *path,
                             uint64_t *first_diff)
{
    if (first_diff) *first_diff = UINT64_MAX;
    if (first > n || count > n - first) return ORACLE_BAD_ARG;
    uint64_t hb = oracle_header_bytes(ts, n), db = oracle_data_bytes(ts, n);
    int fd = open(path, O_RDONLY);
    if (fd < 0) return ORACLE_IO;
    struct stat st;
    if (fstat(fd, &st) != 0) { close(fd); return ORACLE_IO; }
    if ((uint64_t)st.st_size != hb + db) {
        close(fd);
        if (first_diff) *first_diff = (uint64_t)st.st_size < hb + db ? (uint64_t)st.st_size : hb + db;
        return ORACLE_MISMATCH;
    }
    int rc = ORACLE_OK;
    const uint64_t BUF = 8ull << 20;
    uint8_t *buf = (uint8_t *)malloc(BUF);
    if (!buf) { close(fd); return ORACLE_NOMEM; }
    if (first == 0) {
        uint8_t *hdr = (uint8_t *)malloc(hb);
        if (!hdr) { free(buf); close(fd); return ORACLE_NOMEM; }
        rc = oracle_build_header(ts, n, iter, hdr, hb);
        for (uint64_t done = 0; done < hb && rc == ORACLE_OK; ) {
            uint64_t m = hb - done < BUF ? hb - done : BUF;
            rc = read_all(fd, buf, m);
            if (rc == ORACLE_OK && memcmp(buf, hdr + done, m) != 0) {
                uint64_t i = 0;
                while (buf[i] == hdr[done + i]) i++;
                if (first_diff) *first_diff = done + i;
                rc = ORACLE_MISMATCH;
            }
            done += m;
        }
        free(hdr);
    }
    uint64_t pos = oracle_tensor_offset(ts, n, first);
    if (rc == ORACLE_OK && lseek(fd, (off_t)pos, SEEK_SET) != (off_t)pos) rc = ORACLE_IO;
    for (size_t k = first; k < first + count && rc == ORACLE_OK; k++) {
        const uint8_t *src = (const uint8_t *)ts[k].host_bytes;
        if (!src) { rc = ORACLE_BAD_ARG; break; }
        uint64_t padded = round_up(ts[k].nbytes);
        for (uint64_t done = 0; done < padded && rc == ORACLE_OK; ) {
            uint64_t m = padded - done < BUF ? padded - done : BUF;
            rc = read_all(fd, buf, m);
            /* the first `live` bytes of this block are tensor bytes, the rest is padding */
            uint64_t live = done >= ts[k].nbytes ? 0 : (ts[k].nbytes - done < m ? ts[k].nbytes - done : m);
            if (rc == ORACLE_OK) {
                uint64_t i = 0;
                if (memcmp(buf, src + done, live) != 0) { while (buf[i] == src[done + i]) i++; rc = ORACLE_MISMATCH; }
                else for (i = live; i < m; i++) if (buf[i] != 0) { rc = ORACLE_MISMATCH; break; }
                if (rc == ORACLE_MISMATCH && first_diff) *first_diff = pos + i;
            }
            done += m; pos += m;
        }
    }
    free(buf); close(fd);
    return rc;
}

/* Restore: read the file, check it against FORMAT.md's reader checks and against the expected tensor
 * list (names, dtypes, shapes, sizes), then copy each tensor's bytes into host_bytes. The caller
 * moves them to the device with blocking copies. */
int oracle_restore_file(const char *path, oracle_tensor *ts, size_t n, uint64_t *iter_out)
{
    int fd = open(path, O_RDONLY);
    if (fd < 0) return ORACLE_IO;
    struct stat st;
    if (fstat(fd, &st) != 0) { close(fd); return ORACLE_IO; }
    uint8_t fixed[ORACLE_FIXED];
    if ((uint64_t)st.st_size < ORACLE_FIXED || read_all(fd, fixed, ORACLE_FIXED) != ORACLE_OK) { close(fd); return ORACLE_BAD_FILE; }
    uint64_t hb = get_le(fixed + 32, 8), db = get_le(fixed + 40, 8), fb = get_le(fixed + 48, 8);
    if (memcmp(fixed, MAGIC, 8) != 0 || get_le(fixed + 8, 4) != 1 || get_le(fixed + 12, 4) != ORACLE_ALIGN ||
        hb % ORACLE_ALIGN != 0 || hb < ORACLE_FIXED || fb != hb + db || fb != (uint64_t)st.st_size || get_le(fixed + 56, 8) != 0) { close(fd); return ORACLE_BAD_FILE; }
    if (get_le(fixed + 24, 8) != n) { close(fd); return ORACLE_MISMATCH; }
    uint8_t *hdr = (uint8_t *)malloc(hb);
    if (!hdr) { close(fd); return ORACLE_NOMEM; }
    memcpy(hdr, fixed, ORACLE_FIXED);
    int rc = read_all(fd, hdr + ORACLE_FIXED, hb - ORACLE_FIXED);
    const uint8_t *p = hdr + ORACLE_FIXED, *end = hdr + hb;
    uint64_t expect_off = hb;
    for (size_t k = 0; k < n && rc == ORACLE_OK; k++) {
        if (end - p < 2) { rc = ORACLE_BAD_FILE; break; }
        uint64_t len = get_le(p, 2); p += 2;
        if ((uint64_t)(end - p) < len + 2) { rc = ORACLE_BAD_FILE; break; }
        const uint8_t *name = p; p += len;
        int32_t dtype = *p++; uint32_t ndim = *p++;
        if (ndim > 8 || (uint64_t)(end - p) < 8ull * ndim + 16) { rc = ORACLE_BAD_FILE; break; }
        uint64_t numel = 1; int64_t shape[8];
        for (uint32_t d = 0; d < ndim; d++) { shape[d] = (int64_t)get_le(p, 8); p += 8; if (shape[d] < 0) rc = ORACLE_BAD_FILE; else numel *= (uint64_t)shape[d]; }
        uint64_t off = get_le(p, 8); p += 8;
        uint64_t nb = get_le(p, 8); p += 8;
        if (rc != ORACLE_OK) break;
        if (off != expect_off || nb == 0 || nb != elsize(dtype) * numel || off + nb > fb) { rc = ORACLE_BAD_FILE; break; }
        if (len != strlen(ts[k].name) || memcmp(name, ts[k].name, len) != 0 || dtype != ts[k].dtype || ndim != ts[k].ndim || nb != ts[k].nbytes) { rc = ORACLE_MISMATCH; break; }
        for (uint32_t d = 0; d < ndim; d++) if (shape[d] != ts[k].shape[d]) rc = ORACLE_MISMATCH;
        expect_off += round_up(nb);
    }
    if (rc == ORACLE_OK && expect_off != fb) rc = ORACLE_BAD_FILE;
    /* data: sequential read, padding skipped */
    for (size_t k = 0; k < n && rc == ORACLE_OK; k++) {
        if (!ts[k].host_bytes) { rc = ORACLE_BAD_ARG; break; }
        rc = read_all(fd, ts[k].host_bytes, ts[k].nbytes);
        uint64_t pad = round_up(ts[k].nbytes) - ts[k].nbytes;
        if (rc == ORACLE_OK && pad) { uint8_t skip[ORACLE_ALIGN]; rc = read_all(fd, skip, pad); }
    }
    if (rc == ORACLE_OK && iter_out) *iter_out = get_le(fixed + 16, 8);
    free(hdr); close(fd);
    return rc;
}

/* ------------------------------------------------------------------------------------------------
 * Format version 2 (FORMAT.md, "derived tensors"): the data reduction the paper leaves as future work
 * (Conclusions), in its first lossless form. A declared pair (derived d, source s) says: tensor d is the
 * bf16 round-to-nearest-even of f32 tensor s. If every declared pair holds in the captured bytes the file
 * is version 2 and the derived tensors are described but not stored; otherwise it is version 1, as above.
 * ------------------------------------------------------------------------------------------------ */

/* bf16 round-to-nearest-even of an f32 bit pattern, on integers (FORMAT.md). */
uint16_t oracle_bf16_rne(uint32_t u)
{
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);   /* NaN stays NaN, made quiet */
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

static uint32_t load_u32(const uint8_t *p) { return (uint32_t)p[0] | (uint32_t)p[1] << 8 | (uint32_t)p[2] << 16 | (uint32_t)p[3] << 24; }
static uint16_t load_u16(const uint8_t *p) { return (uint16_t)(p[0] | p[1] << 8); }

static int same_shape(const oracle_tensor *a, const oracle_tensor *b)
{
    if (a->ndim != b->ndim) return 0;
    for (uint32_t d = 0; d < a->ndim; d++) if (a->shape[d] != b->shape[d]) return 0;
    return 1;
}

/* A pair list is well formed when every derived tensor is bf16, its source f32 of the same shape, no tensor
 * is derived twice and no source is itself derived. */
static int pairs_ok(const oracle_tensor *ts, size_t n, const uint32_t *derived, const uint32_t *source, size_t n_pairs)
{
    for (size_t i = 0; i < n_pairs; i++) {
        if (derived[i] >= n || source[i] >= n || derived[i] == source[i]) return 0;
        if (ts[derived[i]].dtype != 1 || ts[source[i]].dtype != 2 || !same_shape(&ts[derived[i]], &ts[source[i]])) return 0;
        for (size_t j = 0; j < n_pairs; j++) {
            if (j != i && derived[j] == derived[i]) return 0;
            if (source[j] == derived[i]) return 0;
        }
    }
    return 1;
}

/* 1 when every element of every declared derived tensor equals bf16_rne of its source element, 0 when not;
 * -ORACLE_BAD_ARG for a malformed pair list or missing bytes. Only the tensors named by the pairs need bytes. */
int oracle_pairs_hold(const oracle_tensor *ts, size_t n, const uint32_t *derived, const uint32_t *source, size_t n_pairs)
{
    if (!pairs_ok(ts, n, derived, source, n_pairs)) return -ORACLE_BAD_ARG;
    for (size_t i = 0; i < n_pairs; i++) {
        const uint8_t *p = (const uint8_t *)ts[derived[i]].host_bytes, *m = (const uint8_t *)ts[source[i]].host_bytes;
        if (!p || !m) return -ORACLE_BAD_ARG;
        uint64_t numel = ts[derived[i]].nbytes / 2;
        for (uint64_t e = 0; e < numel; e++)
            if (load_u16(p + 2 * e) != oracle_bf16_rne(load_u32(m + 4 * e))) return 0;
    }
    return 1;
}

/* enc[k] / ref[k] of every tensor for a pair list (caller provides n entries each). */
static void encodings(size_t n, const uint32_t *derived, const uint32_t *source, size_t n_pairs, uint8_t *enc, uint32_t *ref)
{
    for (size_t k = 0; k < n; k++) { enc[k] = 0; ref[k] = 0; }
    for (size_t i = 0; i < n_pairs; i++) { enc[derived[i]] = 1; ref[derived[i]] = source[i]; }
}

static uint64_t v2_header_bytes(const oracle_tensor *ts, size_t n)
{
    uint64_t used = ORACLE_FIXED;
    for (size_t k = 0; k < n; k++) used += entry_len(&ts[k]) + 1 + 4;
    return round_up(used);
}

static uint64_t v2_data_bytes(const oracle_tensor *ts, size_t n, const uint8_t *enc)
{
    uint64_t total = 0;
    for (size_t k = 0; k < n; k++) if (!enc[k]) total += round_up(ts[k].nbytes);
    return total;
}

/* Sizes of the version-2 file of a tensor list with the given pairs (header, data). */
int oracle_v2_sizes(const oracle_tensor *ts, size_t n, const uint32_t *derived, const uint32_t *source, size_t n_pairs,
                    uint64_t *header_bytes, uint64_t *data_bytes)
{
    if (!pairs_ok(ts, n, derived, source, n_pairs)) return ORACLE_BAD_ARG;
    uint8_t *enc = (uint8_t *)malloc(n ? n : 1);
    uint32_t *ref = (uint32_t *)malloc((n ? n : 1) * sizeof *ref);
    if (!enc || !ref) { free(enc); free(ref); return ORACLE_NOMEM; }
    encodings(n, derived, source, n_pairs, enc, ref);
    if (header_bytes) *header_bytes = v2_header_bytes(ts, n);
    if (data_bytes) *data_bytes = v2_data_bytes(ts, n, enc);
    free(enc); free(ref);
    return ORACLE_OK;
}

static int v2_build_header(const oracle_tensor *ts, size_t n, const uint8_t *enc, const uint32_t *ref, uint64_t iter, uint8_t *out, uint64_t cap)
{
    for (size_t k = 0; k < n; k++) if (!tensor_ok(&ts[k])) return ORACLE_BAD_ARG;
    uint64_t hb = v2_header_bytes(ts, n), db = v2_data_bytes(ts, n, enc);
    if (cap < hb) return ORACLE_BAD_ARG;
    memset(out, 0, hb);
    memcpy(out, MAGIC, 8);
    put_le(out + 8, 2, 4);
    put_le(out + 12, ORACLE_ALIGN, 4);
    put_le(out + 16, iter, 8);
    put_le(out + 24, n, 8);
    put_le(out + 32, hb, 8);
    put_le(out + 40, db, 8);
    put_le(out + 48, hb + db, 8);
    uint8_t *p = out + ORACLE_FIXED;
    uint64_t off = hb;
    for (size_t k = 0; k < n; k++) {
        size_t len = strlen(ts[k].name);
        put_le(p, len, 2); p += 2;
        memcpy(p, ts[k].name, len); p += len;
        *p++ = (uint8_t)ts[k].dtype;
        *p++ = (uint8_t)ts[k].ndim;
        for (uint32_t d = 0; d < ts[k].ndim; d++) { put_le(p, (uint64_t)ts[k].shape[d], 8); p += 8; }
        put_le(p, enc[k] ? 0 : off, 8); p += 8;
        put_le(p, ts[k].nbytes, 8); p += 8;
        *p++ = enc[k];
        put_le(p, ref[k], 4); p += 4;
        if (!enc[k]) off += round_up(ts[k].nbytes);
    }
    return ORACLE_OK;
}

/* The serializer with declared pairs, into memory: version 2 when the pairs hold, else exactly the version-1
 * file. *version_out says which; *written its size. cap must cover the version-1 size (the larger one). */
int oracle_v2_serialize_mem(const oracle_tensor *ts, size_t n, const uint32_t *derived, const uint32_t *source, size_t n_pairs,
                            uint64_t iter, uint8_t *out, uint64_t cap, uint64_t *written, uint32_t *version_out)
{
    int hold = oracle_pairs_hold(ts, n, derived, source, n_pairs);
    if (hold < 0) return -hold;
    if (!hold || n_pairs == 0) {
        if (version_out) *version_out = 1;
        return oracle_serialize_mem(ts, n, iter, out, cap, written);
    }
    uint8_t *enc = (uint8_t *)malloc(n);
    uint32_t *ref = (uint32_t *)malloc(n * sizeof *ref);
    if (!enc || !ref) { free(enc); free(ref); return ORACLE_NOMEM; }
    encodings(n, derived, source, n_pairs, enc, ref);
    uint64_t hb = v2_header_bytes(ts, n), db = v2_data_bytes(ts, n, enc);
    int rc = cap < hb + db ? ORACLE_BAD_ARG : v2_build_header(ts, n, enc, ref, iter, out, cap);
    uint8_t *p = out + hb;
    for (size_t k = 0; k < n && rc == ORACLE_OK; k++) {
        if (enc[k]) continue;
        if (!ts[k].host_bytes) { rc = ORACLE_BAD_ARG; break; }
        uint64_t padded = round_up(ts[k].nbytes);
        memcpy(p, ts[k].host_bytes, ts[k].nbytes);
        memset(p + ts[k].nbytes, 0, padded - ts[k].nbytes);
        p += padded;
    }
    if (rc == ORACLE_OK) { if (written) *written = hb + db; if (version_out) *version_out = 2; }
    free(enc); free(ref);
    return rc;
}

/* Piecewise comparison of a file that is expected to be version `version` (1: oracle_compare_file_span on the
 * same arguments; 2: derived tensors occupy no bytes). Tensors [first, first+count) need bytes unless derived. */
int oracle_v2_compare_file_span(const oracle_tensor *ts, size_t n, const uint32_t *derived, const uint32_t *source, size_t n_pairs,
                                uint32_t version, uint64_t iter, size_t first, size_t count, const char *path, uint64_t *first_diff)
{
    if (version == 1) return oracle_compare_file_span(ts, n, iter, first, count, path, first_diff);
    if (first_diff) *first_diff = UINT64_MAX;
    if (version != 2 || first > n || count > n - first || !pairs_ok(ts, n, derived, source, n_pairs)) return ORACLE_BAD_ARG;
    uint8_t *enc = (uint8_t *)malloc(n ? n : 1);
    uint32_t *ref = (uint32_t *)malloc((n ? n : 1) * sizeof *ref);
    const uint64_t BUF = 8ull << 20;
    uint8_t *buf = (uint8_t *)malloc(BUF);
    if (!enc || !ref || !buf) { free(enc); free(ref); free(buf); return ORACLE_NOMEM; }
    encodings(n, derived, source, n_pairs, enc, ref);
    uint64_t hb = v2_header_bytes(ts, n), db = v2_data_bytes(ts, n, enc);
    int rc = ORACLE_OK;
    int fd = open(path, O_RDONLY);
    struct stat st;
    if (fd < 0 || fstat(fd, &st) != 0) rc = ORACLE_IO;
    else if ((uint64_t)st.st_size != hb + db) {
        if (first_diff) *first_diff = (uint64_t)st.st_size < hb + db ? (uint64_t)st.st_size : hb + db;
        rc = ORACLE_MISMATCH;
    }
    if (rc == ORACLE_OK && first == 0) {
        uint8_t *hdr = (uint8_t *)malloc(hb), *got = (uint8_t *)malloc(hb);
        if (!hdr || !got) rc = ORACLE_NOMEM;
        if (rc == ORACLE_OK) rc = v2_build_header(ts, n, enc, ref, iter, hdr, hb);
        if (rc == ORACLE_OK) rc = read_all(fd, got, hb);
        if (rc == ORACLE_OK && memcmp(got, hdr, hb) != 0) {
            uint64_t i = 0;
            while (got[i] == hdr[i]) i++;
            if (first_diff) *first_diff = i;
            rc = ORACLE_MISMATCH;
        }
        free(hdr); free(got);
    }
    uint64_t pos = hb;
    for (size_t k = 0; k < first; k++) if (!enc[k]) pos += round_up(ts[k].nbytes);
    if (rc == ORACLE_OK && lseek(fd, (off_t)pos, SEEK_SET) != (off_t)pos) rc = ORACLE_IO;
    for (size_t k = first; k < first + count && rc == ORACLE_OK; k++) {
        if (enc[k]) continue;
        const uint8_t *src = (const uint8_t *)ts[k].host_bytes;
        if (!src) { rc = ORACLE_BAD_ARG; break; }
        uint64_t padded = round_up(ts[k].nbytes);
        for (uint64_t done = 0; done < padded && rc == ORACLE_OK; ) {
            uint64_t m = padded - done < BUF ? padded - done : BUF;
            rc = read_all(fd, buf, m);
            uint64_t live = done >= ts[k].nbytes ? 0 : (ts[k].nbytes - done < m ? ts[k].nbytes - done : m);
            if (rc == ORACLE_OK) {
                uint64_t i = 0;
                if (memcmp(buf, src + done, live) != 0) { while (buf[i] == src[done + i]) i++; rc = ORACLE_MISMATCH; }
                else for (i = live; i < m; i++) if (buf[i] != 0) { rc = ORACLE_MISMATCH; break; }
                if (rc == ORACLE_MISMATCH && first_diff) *first_diff = pos + i;
            }
            done += m; pos += m;
        }
    }
    if (fd >= 0) close(fd);
    free(enc); free(ref); free(buf);
    return rc;
}

/* Restore with declared pairs: a version-1 file goes through oracle_restore_file; a version-2 file must carry
 * exactly the declared pairs as derived entries, its stored tensors are read in order and every derived tensor
 * is recomputed from its restored source. All n tensors need writable host_bytes. */
int oracle_v2_restore_file(const char *path, oracle_tensor *ts, size_t n, const uint32_t *derived, const uint32_t *source, size_t n_pairs,
                           uint64_t *iter_out, uint32_t *version_out)
{
    if (!pairs_ok(ts, n, derived, source, n_pairs)) return ORACLE_BAD_ARG;
    int fd = open(path, O_RDONLY);
    if (fd < 0) return ORACLE_IO;
    struct stat st;
    uint8_t fixed[ORACLE_FIXED];
    if (fstat(fd, &st) != 0 || (uint64_t)st.st_size < ORACLE_FIXED || read_all(fd, fixed, ORACLE_FIXED) != ORACLE_OK) { close(fd); return ORACLE_BAD_FILE; }
    if (memcmp(fixed, MAGIC, 8) == 0 && get_le(fixed + 8, 4) == 1) {
        close(fd);
        if (version_out) *version_out = 1;
        return oracle_restore_file(path, ts, n, iter_out);
    }
    uint64_t hb = get_le(fixed + 32, 8), db = get_le(fixed + 40, 8), fb = get_le(fixed + 48, 8);
    if (memcmp(fixed, MAGIC, 8) != 0 || get_le(fixed + 8, 4) != 2 || get_le(fixed + 12, 4) != ORACLE_ALIGN || hb % ORACLE_ALIGN != 0 ||
        hb < ORACLE_FIXED || fb != hb + db || fb != (uint64_t)st.st_size || get_le(fixed + 56, 8) != 0) { close(fd); return ORACLE_BAD_FILE; }
    if (get_le(fixed + 24, 8) != n) { close(fd); return ORACLE_MISMATCH; }
    uint8_t *hdr = (uint8_t *)malloc(hb), *enc = (uint8_t *)malloc(n ? n : 1);
    uint32_t *ref = (uint32_t *)malloc((n ? n : 1) * sizeof *ref);
    if (!hdr || !enc || !ref) { free(hdr); free(enc); free(ref); close(fd); return ORACLE_NOMEM; }
    encodings(n, derived, source, n_pairs, enc, ref);
    int rc = read_all(fd, hdr + ORACLE_FIXED, hb - ORACLE_FIXED);
    const uint8_t *p = hdr + ORACLE_FIXED, *end = hdr + hb;
    uint64_t expect_off = hb;
    for (size_t k = 0; k < n && rc == ORACLE_OK; k++) {
        if (end - p < 2) { rc = ORACLE_BAD_FILE; break; }
        uint64_t len = get_le(p, 2); p += 2;
        if ((uint64_t)(end - p) < len + 2) { rc = ORACLE_BAD_FILE; break; }
        const uint8_t *name = p; p += len;
        int32_t dtype = *p++; uint32_t ndim = *p++;
        if (ndim > 8 || (uint64_t)(end - p) < 8ull * ndim + 16 + 5) { rc = ORACLE_BAD_FILE; break; }
        uint64_t numel = 1; int64_t shape[8];
        for (uint32_t d = 0; d < ndim; d++) { shape[d] = (int64_t)get_le(p, 8); p += 8; if (shape[d] < 0) rc = ORACLE_BAD_FILE; else numel *= (uint64_t)shape[d]; }
        uint64_t off = get_le(p, 8); p += 8;
        uint64_t nb = get_le(p, 8); p += 8;
        uint32_t e = *p++;
        uint32_t r = (uint32_t)get_le(p, 4); p += 4;
        if (rc != ORACLE_OK) break;
        if (e > 1 || nb == 0 || nb != elsize(dtype) * numel) { rc = ORACLE_BAD_FILE; break; }
        if (e == 0 && (off != expect_off || off + nb > fb || r != 0)) { rc = ORACLE_BAD_FILE; break; }
        if (e == 1 && (off != 0 || dtype != 1 || r >= n)) { rc = ORACLE_BAD_FILE; break; }
        if (len != strlen(ts[k].name) || memcmp(name, ts[k].name, len) != 0 || dtype != ts[k].dtype || ndim != ts[k].ndim || nb != ts[k].nbytes ||
            e != enc[k] || r != ref[k]) { rc = ORACLE_MISMATCH; break; }
        for (uint32_t d = 0; d < ndim; d++) if (shape[d] != ts[k].shape[d]) rc = ORACLE_MISMATCH;
        if (e == 0) expect_off += round_up(nb);
    }
    if (rc == ORACLE_OK && expect_off != fb) rc = ORACLE_BAD_FILE;
    for (size_t k = 0; k < n && rc == ORACLE_OK; k++) {
        if (!ts[k].host_bytes) { rc = ORACLE_BAD_ARG; break; }
        if (enc[k]) continue;
        rc = read_all(fd, ts[k].host_bytes, ts[k].nbytes);
        uint64_t pad = round_up(ts[k].nbytes) - ts[k].nbytes;
        if (rc == ORACLE_OK && pad) { uint8_t skip[ORACLE_ALIGN]; rc = read_all(fd, skip, pad); }
    }
    for (size_t i = 0; i < n_pairs && rc == ORACLE_OK; i++) {
        uint8_t *d = (uint8_t *)ts[derived[i]].host_bytes;
        const uint8_t *m = (const uint8_t *)ts[source[i]].host_bytes;
        uint64_t numel = ts[derived[i]].nbytes / 2;
        for (uint64_t e = 0; e < numel; e++) put_le(d + 2 * e, oracle_bf16_rne(load_u32(m + 4 * e)), 2);
    }
    if (rc == ORACLE_OK && iter_out) *iter_out = get_le(fixed + 16, 8);
    if (rc == ORACLE_OK && version_out) *version_out = 2;
    free(hdr); free(enc); free(ref); close(fd);
    return rc;
}
