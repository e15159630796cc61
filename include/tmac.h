/*
 * tmac.h -- C ABI of the MI355X (gfx950) LUT-based mixed-precision GEMV/GEMM library.
 *
 * The library computes R[N,M] = A[N,K] x W[M,K]^T for b-bit (b = 1..4) group-quantised
 * weights W without ever de-quantising them, by the table-lookup method of T-MAC
 * (arxiv 2407.00088): weights are split into b one-bit planes (Eq. 1), every g = 4
 * consecutive bits of a plane along K form a 4-bit index (Algorithm 1,
 * PreprocessWeights), every group of g activations is expanded into a table of 2^g
 * signed partial sums (Algorithm 1, Precompute; Section 3.1), and the product is the
 * sum of looked-up table entries, shifted by the plane's weight 2^i, plus a bias term
 * (Algorithm 1, main loop; Section 4 "Bit-serial linear transformation" with
 * s0 = -1, s1 = +1, i.e. alpha_i = beta_i = 1/2).
 *
 * De-quantisation convention (the paper only speaks of "quantization scales"; the
 * zero point is this library's reading): w[m,k] = s[m,k/G] * (q[m,k] - z[m,k/G]),
 * q an unsigned b-bit code, s and z fp16, z real-valued in code units.
 *
 * Result:  R[n,m] = sum_G s[m,G] * ( 1/2 * sum_i 2^i L_i[n,m,G] + ((2^b-1)/2 - z[m,G]) * S[n,G] )
 *   L_i[n,m,G] = sum over the LUT groups kg of quantisation group G of T[n,kg,idx_i[m,kg]]
 *   S[n,G]     = sum of the activations of quantisation group G.
 *
 * General rules
 *   - The library allocates no memory; the caller owns every buffer.  The only state it keeps is
 *     the text of the calling thread's last error (tmac_last_error_detail) and, once
 *     tmac_mpgemm_noalloc has run on a GPU, that GPU's address of the library's scratch array.
 *   - Pointers named *_host are host memory, *_dev are device memory of the current HIP device.
 *     Device pointers must be 16-byte aligned (256 recommended).
 *   - Device entry points only enqueue work on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and never synchronise.
 *   - Every failure is reported through the returned tmac_status; arguments are checked on
 *     the host before anything is launched, and nothing is launched when a check fails.
 *   - Only gfx950 code objects are built into the library.
 */
#ifndef TMAC_H_
#define TMAC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TMAC_OK = 0,
  TMAC_EINVAL = 1,        /* null/misaligned pointer, bad enum, shape constraint violated   */
  TMAC_EUNSUPPORTED = 2,  /* valid request that this build has no kernel for                 */
  TMAC_ESIZE = 3,         /* a caller-provided buffer is too small                           */
  TMAC_EHIP = 4           /* the HIP runtime reported an error while enqueuing               */
} tmac_status;

/* Activation type.  TMAC_ACT_F16_TQ is accepted by the calls that build their tables inside the
 * lookup kernel (tmac_mpgemv_fused, tmac_mpgemv_fused_ex, tmac_mpgemv_fused_multi, and
 * tmac_mpgemm_fused where it is one of those): fp16 activations whose tables are quantised to int8
 * in the kernel, i.e. the arithmetic of TMAC_LUT_I8Q without a LUT buffer. */
typedef enum { TMAC_ACT_F16 = 0, TMAC_ACT_I8 = 1, TMAC_ACT_F16_TQ = 2 } tmac_act_t;

/* Table entry type.
 *   TMAC_LUT_F16: entries are signed sums of fp16 activations formed with fp16 additions (see
 *                 tmac_precompute_lut; results within 2e-3 relative Frobenius error of the fp64
 *                 product).
 *   TMAC_LUT_I16: entries are exact int16 sums of int8 activations (|T| <= 4*127); all
 *                 aggregation is int32 and the result is bit-exact.
 *   TMAC_LUT_I8Q: table quantisation (Section 3.3): entries of fp16 activations' tables rounded
 *                 to int8 with one dynamic scale per 16 activations (four tables),
 *                 scale = max|T| / 127; the look-ups of those four tables are added as
 *                 integers and multiplied by the scale once.  Lossy (about 4e-3 relative
 *                 error on Gaussian data); packed layout 2 only.  With a LUT buffer for at most
 *                 64 activation rows; the fused calls quantise the tables in the kernel
 *                 (TMAC_ACT_F16_TQ) for any N. */
typedef enum { TMAC_LUT_F16 = 0, TMAC_LUT_I16 = 1, TMAC_LUT_I8Q = 2 } tmac_lut_t;

/* TMAC_OUT_I32 (raw integer dot products) is available with TMAC_LUT_I16 and a
 * per-tensor scale (group == 0) with an integer zero point only. */
typedef enum { TMAC_OUT_F32 = 0, TMAC_OUT_F16 = 1, TMAC_OUT_I32 = 2 } tmac_out_t;

/* Weight matrix description (Algorithm 1: W has shape [M, K]).
 *   bits   1..4, weight bit-width b
 *   g      LUT group size: 4 (one 16-entry table per 4 activations, the paper's choice) in both
 *          layouts; layout 3 also takes 2 and 8 (4- and 256-entry tables: Section 4 discusses
 *          how g trades table size against the number of look-ups); K % g == 0
 *   group  quantisation group G along K (which sizes a layout accepts is said with the layout);
 *          == K: one scale per row; 0 = one scale and zero for the whole tensor
 *   layout TMAC_LAYOUT_*: 2 is the decode layout (few activation rows: up to about 8), 3 serves
 *          any number of activation rows and is the fast one from about 16 on
 *   zero_point  per-tensor zero in code units (group == 0 only), e.g. 1 for ternary
 *          weights stored as q = t+1 (Section 5.1: ternary weights run as 2-bit) */
typedef struct {
  int32_t M, K, bits, g, group, layout;
  float   zero_point;   /* zero point of the whole tensor, used when group == 0 */
  int32_t reserved;     /* must be 0 */
} tmac_wdesc;

/* A packed blob is a 256-byte header (struct tmac_blob_header below), the index region and the
 * scale/zero region, each starting at a multiple of 256 bytes.  Rows >= M and k >= K are padded
 * with index 0.  Bit (k % 4) of a 4-bit index belongs to element k (lowest k = least significant
 * bit).  K is padded to a multiple of 128 (Kp).
 *
 * Packed layout 2 ("tile 8 rows x units of 16 k", for the register-table decode kernel;
 * Section 3.2 permutation + interleaving, Section 3.3 mirror consolidation folded into
 * the stored indices):
 *
 *   header   Mp = M rounded up to 8, n_tiles = Mp/8, n_chunks = Kp/16 units
 *   indices  per tile t (rows 8t..8t+7) the records of its n_units units, 4*bits dwords each:
 *            record[tb][d], unit u = k in [16u, 16u+16), table tb = LUT group kg = 4u + tb.
 *            One lane of the kernel owns one unit (four tables held in registers).  Eight
 *            consecutive units form a chunk of 128 k; the n_units/8 chunks of a row are split
 *            into nB = ceil(chunks/8) consecutive blocks, the first chunks % nB of them with
 *            floor(chunks/nB) + 1 chunks, the others with floor(chunks/nB); one block per
 *            wavefront pass.  Inside a block of ng chunks starting at chunk c0, unit
 *            8*(c0 + j) + pos (j < ng, pos < 8) belongs to lane 8*pos + j and sits in slot
 *            s = pos*ng + j; the records are stored piece-major: the 16-byte piece i (dwords
 *            4i..4i+3 of the flattened record) of slot s sits at dword offset
 *            (t*n_units + 8*c0)*4*bits + (i*8*ng + s)*4, so that each of the `bits` load
 *            instructions of a wavefront reads one contiguous run, and the eight lanes that
 *            share (lane & 7) cover one chunk.
 *            Stored 4-bit code of an index p:  p < 8 ? p : 8 | (15 - p)   (bit 3 = negate,
 *            bits 0..2 = entry of the stored half table, because T[p] = -T[15-p]).
 *            Byte y of a dword holds two codes of the same table, one for the "low" row and
 *            one for the "high" row: bits 0..2 = entry of the low row's code, bit 7 = its negate
 *            bit; bits 4..6 = entry of the high row's code, whose negate bit sits in bit 3 of
 *            byte (y + 1) mod 4 of the same dword (rotated right by four bits, the dword shows
 *            the high rows' codes as it shows the low rows' unrotated).  With r = row in tile:
 *              bits = 4: dword d = 0..3:  low = (r = 2d, plane y), high = (r = 2d+1, plane y)
 *              bits = 2: dword d = 0..1:  low = (r = 4d + y/2, plane y%2),
 *                                         high = (r = 4d + 2 + y/2, plane y%2)
 *              bits = 1: dword 0:         low = (r = y, plane 0), high = (r = 4 + y, plane 0)
 *              bits = 3: dwords 0,1 as bits = 2 (planes 0,1); dword 2 as bits = 1 with plane 2
 *   scales   u16 sz[n_tiles][n_qgroups][8][2] = {fp16 scale, fp16 zero}
 *   Group sizes: any multiple of 16, or K, or 0 (per tensor).
 */
/* Packed layout 3 ("tile 64 rows x chunks of 32 k", for the batched lookup kernel that serves many
 * activation rows; Section 3.2: a large tile over M lets many weight rows reuse one table):
 *
 *   header   Mp = M rounded up to 64, n_tiles = Mp/64, n_chunks = Kp/32
 *   indices  u32 idx[n_tiles][n_chunks][64][bits]: dword [t][c][r][i] holds the eight 4-bit
 *            indices of bit plane i of row 64t+r for LUT groups kg = 8c + j, index j in nibble j
 *            (bits 4j..4j+3).  One lane of the kernel owns one row and reads its `bits` dwords of
 *            a chunk with one load; (x << 3) & 0x78787878 and (x >> 1) & 0x78787878 are the
 *            byte offsets of the even and odd tables' entries.  Bit t of the dword is bit plane
 *            i of q[64t+r][32c+t], so the same dword read as sixteen 2-bit or four 8-bit fields
 *            holds the indices for g = 2 or g = 8: the index region does not depend on g.
 *   scales   u16 sz[n_tiles][n_qgroups][64][2] = {fp16 scale, fp16 zero}
 *   Group sizes: any multiple of 32, or K, or 0 (per tensor).  Table types: TMAC_LUT_F16 and
 *   TMAC_LUT_I16.
 */
enum { TMAC_LAYOUT_R8U16 = 2, TMAC_LAYOUT_R64K32 = 3 };

typedef struct {
  uint32_t magic;        /* 0x43414D54 "TMAC" */
  uint32_t layout;
  int32_t  M, K, bits, g, group;
  int32_t  Mp, Kp;       /* M rounded up to the layout's row tile, K rounded up to 128 */
  int32_t  n_tiles, n_chunks, n_qgroups;
  float    zero_point;   /* per-tensor zero (group == 0) */
  uint32_t reserved0;
  uint64_t idx_off, idx_bytes, sz_off, sz_bytes, total_bytes;
  uint8_t  pad[256 - 14 * 4 - 5 * 8];
} tmac_blob_header;

/* Size in bytes of the packed blob for `desc`, header included; 0 if `desc` is invalid. */
size_t tmac_packed_bytes(const tmac_wdesc* desc);

/* Offline weight preparation (Algorithm 1 PreprocessWeights; Section 3.2 permutation and
 * interleaving).  Host to host; the caller uploads the blob to the device afterwards.
 *   q_host       [M,K] row-major, one unsigned code per byte, each < 2^bits
 *   scales_host  fp16 bits, [M, K/G] row-major (ignored when group == 0: the per-tensor
 *                scale is given to tmac_mpgemm)
 *   zeros_host   fp16 bits, [M, K/G] row-major; NULL means z = (2^b-1)/2 (symmetric
 *                levels, the bias term vanishes); ignored when group == 0 (the zero of
 *                the whole tensor is desc->zero_point)
 *   packed_host  output, packed_bytes >= tmac_packed_bytes(desc)
 * The device entry points do not read the blob on the host: passing a blob packed for a different
 * desc to them is undefined; tmac_blob_check compares a host copy of the header with a desc.
 * Errors: TMAC_EINVAL (null pointer, bad desc, code out of range), TMAC_ESIZE. */
tmac_status tmac_pack_weights(const tmac_wdesc* desc, const uint8_t* q_host,
                              const uint16_t* scales_host, const uint16_t* zeros_host,
                              void* packed_host, size_t packed_bytes);

/* Bytes of the LUT buffer for N activation rows.  The tables of the batched kernels come first,
 * laid out as those kernels keep them in LDS: [n tile][Kp/g][2^g][NT] 16-bit entries, where an
 * n tile is NT consecutive activation rows (NT = 4 for N <= 4, for g = 8, and when N % 8 is 1..4
 * below N = 40; else 8; rows that pad the last tile hold zeros) and the NT values of an entry sit
 * side by side; all-zero tables in the k padding.  g = 2 or 8 (16-bit table types only): then
 * the group sums S[N][n_qgroups], 256-byte aligned.  g = 4: these tables (k
 * padded to 128 with all-zero tables; absent for TMAC_LUT_I8Q, which has unit scales [N][Kp/16]
 * and one-byte half tables instead), then the group sums S[N][n_qgroups], then the sums
 * of every 16 consecutive activations S16[N][Kp/16] (both fp32 for TMAC_LUT_F16, int32 for
 * TMAC_LUT_I16), the sums of every 128 consecutive activations S128[N][Kp/128] (same type) and
 * the mirror-consolidated byte-split half tables of the register-table kernel, each region
 * 256-byte aligned.  The three regions of the register-table kernel exist up to N = 64 (beyond
 * that tmac_mpgemm returns TMAC_EUNSUPPORTED for layout 2; its fused call takes any N).
 * The size is therefore not monotonic in N (64 rows need more than 65): a buffer shared by calls
 * of different N takes the largest of their sizes.  The layout inside the buffer belongs to the
 * N it was filled for.  0 on bad arguments. */
size_t tmac_lut_bytes(int32_t N, int32_t K, int32_t g, int32_t group, tmac_lut_t lut);

/* Online table precompute (Algorithm 1 Precompute; Section 3.1; mirror consolidation of
 * Section 3.3 is used to compute half of the entries and negate them for the rest):
 *   T[n,kg,p] = sum_{j<g} (bit j of p ? +a : -a)[n, g*kg+j],  S[n,G] = sum_{k in G} a[n,k].
 * fp16 tables are built in fp16 arithmetic: the g signed terms are added pairwise,
 * ((+-a0 +- a1) + (+-a2 +- a3)) + ..., every addition rounded to nearest even (one addition at
 * g = 2, three levels at g = 8); the kernels that build their tables themselves take the same
 * additions, so both routes give the same bits.  Integer tables are exact.  S is summed in fp32
 * (int32).  int8 tables (TMAC_LUT_I8Q) are quantised from fp32 sums.
 *   A_dev  [N,K] row-major with leading dimension lda (elements): fp16 or int8
 *   TMAC_ACT_F16 goes with TMAC_LUT_F16 or TMAC_LUT_I8Q, TMAC_ACT_I8 with TMAC_LUT_I16.
 * Errors: TMAC_EINVAL, TMAC_ESIZE, TMAC_EHIP. */
tmac_status tmac_precompute_lut(const void* A_dev, tmac_act_t act, int32_t N, int32_t K,
                                int64_t lda, int32_t g, int32_t group, tmac_lut_t lut,
                                void* lut_dev, size_t lut_bytes, void* stream);

/* Bytes of workspace tmac_mpgemm needs for exactly N activation rows (split-K partial sums; how
 * a call is split depends on N, so a buffer meant for several N must take the largest).  Its
 * contents need not be initialised and mean nothing between calls.  Calls that share a workspace
 * must not overlap in time. */
size_t tmac_workspace_bytes(const tmac_wdesc* desc, int32_t N);

/* Look-up, bit-plane shift-accumulate, scale/zero, reduce (Algorithm 1 main loop, Eq. 1,
 * Section 4 bit-serial linear transformation).
 *   packed_dev     blob written by tmac_pack_weights, uploaded unchanged
 *   lut_dev        buffer filled by tmac_precompute_lut with the same N, K, group, lut
 *   act_scale_dev  fp32 [N] per-row activation scale, multiplied into the result
 *                  (TMAC_LUT_I16 path); NULL = 1
 *   weight_scale   per-tensor weight scale, used when desc->group == 0
 *   out_dev        R[N,M] row-major with leading dimension ldo (elements)
 * Integer path result (group == 0, integer zero): R_int = sum_k a_q[n,k]*(q[m,k]-z) exactly;
 * TMAC_OUT_I32 stores R_int, TMAC_OUT_F32 stores fl(fl(float(R_int)*act_scale[n])*weight_scale).
 * The fp reduction order is fixed, so results are reproducible run to run.
 * Errors: TMAC_EINVAL, TMAC_EUNSUPPORTED, TMAC_ESIZE, TMAC_EHIP. */
tmac_status tmac_mpgemm(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev,
                        tmac_lut_t lut, int32_t N, const float* act_scale_dev,
                        float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                        void* workspace_dev, size_t workspace_bytes, void* stream);

/* Decode call with the table precompute fused into the lookup kernel (Algorithm 1 Precompute
 * and main loop in one launch; Section 3.1: the tables are small and cheap to build, so every
 * lane rebuilds the four tables of its 16 activations in registers instead of reading them from
 * a LUT buffer).  Same result as tmac_precompute_lut + tmac_mpgemm on a layout-2 blob: table
 * entries, chunk sums and summation order are identical for group sizes that are multiples
 * of 16.
 *   packed_dev  layout-2 (TMAC_LAYOUT_R8U16) blob; K must be a multiple of 16
 *   A_dev       [N,K] fp16 (TMAC_ACT_F16: fp16 tables; TMAC_ACT_F16_TQ: int8 tables quantised in
 *               the kernel, Section 3.3, the same entries and scales as tmac_precompute_lut with
 *               TMAC_LUT_I8Q up to the last bit of the fp32 sums they are rounded from) or int8
 *               (TMAC_ACT_I8: exact integer tables), 16-byte aligned, leading dimension lda a
 *               multiple of 8 (fp16) or 16 (int8)
 *   other arguments as tmac_mpgemm; no LUT buffer and no workspace.
 * Errors: TMAC_EINVAL, TMAC_EUNSUPPORTED (layout 3, K % 16 != 0, unsupported group), TMAC_EHIP. */
tmac_status tmac_mpgemv_fused(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                              tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                              float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                              void* stream);

/* One call for either layout and any N: the result of tmac_precompute_lut followed by
 * tmac_mpgemm (fp16 tables for TMAC_ACT_F16, exact integer tables for TMAC_ACT_I8), computed
 * from the activations.  The tables are built inside the lookup kernel where a kernel does that
 * (Algorithm 1 Precompute next to the look-ups that use it: no second launch and no table
 * traffic): layout 2 with K % 16 == 0 (this is then tmac_mpgemv_fused), and layout 3 with g = 4,
 * K % 8 == 0, a group size that divides 256 (or one scale per row or tensor), and at most 32
 * activation rows in a call that is cut into K slices of 256 (the case a separate precompute
 * launch costs most).  Every other call
 * runs tmac_precompute_lut into the second region of the workspace and tmac_mpgemm after it
 * (layout 2 with K % 16 != 0 or an unsupported group size: at most 64 activation rows, beyond
 * that TMAC_EUNSUPPORTED and a size of 0).
 *   A_dev          [N,K] fp16 or int8, 16-byte aligned; leading dimension lda a multiple of 8
 *                  where the tables are built in the kernel (16 for int8 with layout 2), else as
 *                  for tmac_precompute_lut
 *   workspace_dev  tmac_fused_workspace_bytes(desc, N, act) bytes, 16-byte aligned, contents
 *                  arbitrary (its first region is tmac_mpgemm's workspace); calls that share it
 *                  must not overlap in time
 * Errors: TMAC_EINVAL, TMAC_EUNSUPPORTED, TMAC_ESIZE, TMAC_EHIP. */
size_t tmac_fused_workspace_bytes(const tmac_wdesc* desc, int32_t N, tmac_act_t act);
tmac_status tmac_mpgemm_fused(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                              tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                              float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                              void* workspace_dev, size_t workspace_bytes, void* stream);

/* Launch-shape knobs of the register-table kernel (layout 2) for benchmarking sweeps; 0 = library
 * default; all must be 0 for layout 3 (TMAC_EUNSUPPORTED otherwise).  Results do not depend on
 * rows_per_group or workgroup_waves; group_waves changes the order in which partial sums over K are
 * added (every setting is deterministic and within the same error bound).
 *   rows_per_group   weight rows that share one set of tables: 8 or 16 (default: 8, and 16 once a
 *                    call has more than about 8000 wavefronts, where sharing the tables pays)
 *   group_waves      most wavefronts that split the K of one group of rows, 1..16 (default 8); a
 *                    row of K elements has ceil(K / 1024) blocks, dealt round-robin to the group's waves
 *   workgroup_waves  wavefronts per workgroup, 1..16, rounded down to whole groups (at least one)
 *   workgroups_per_cu  most workgroups resident on one compute unit, 2..8 (enforced by asking for
 *                    LDS that nobody uses; default: whatever registers and wave slots allow) */
typedef struct {
  int32_t rows_per_group, group_waves, workgroup_waves, workgroups_per_cu, reserved[4];
} tmac_tuning;

/* Same as tmac_mpgemm with explicit launch-shape knobs (NULL = defaults). */
tmac_status tmac_mpgemm_ex(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev,
                           tmac_lut_t lut, int32_t N, const float* act_scale_dev,
                           float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                           void* workspace_dev, size_t workspace_bytes, void* stream,
                           const tmac_tuning* tuning);

/* Same as tmac_mpgemv_fused with explicit launch-shape knobs (NULL = defaults; only
 * rows_per_group applies). */
tmac_status tmac_mpgemv_fused_ex(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                                 tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                                 float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                 void* stream, const tmac_tuning* tuning);

/* Several independent decode GEMVs in ONE launch (the paper's end-to-end section, 5.3, shows that
 * what surrounds the kernels eats their gains: a decode GEMV of a few megabytes costs about as
 * much to launch as to run).  Item i is the call tmac_mpgemv_fused(desc, packed_dev, A_dev, act, N,
 * lda, act_scale_dev, weight_scale, out_dev, out, ldo, stream); the workgroups of one grid are
 * dealt out over the row tiles of all matrices, tables are built inside the kernel as in the single
 * call, and the result of every item equals that single call's bit for bit (the summation order of
 * a matrix does not depend on what else is in the launch).
 *   items   host array of `count` items, 1 <= count <= TMAC_MULTI_MAX; read before the call returns
 *   every desc: layout 2, K % 16 == 0, the same bits; the scales of all matrices must be grouped
 *   the same way (all per row or per tensor, or all with group sizes that are multiples of 128, or
 *   all with other multiples of 16); M, K, group size, pointers and leading dimensions are per item.
 *   act, N, out are common to the items.  Items must not alias each other's outputs.
 *   tuning  NULL = defaults (only rows_per_group applies)
 * Errors: TMAC_EINVAL (null or misaligned pointer, bad desc or leading dimension),
 * TMAC_EUNSUPPORTED (count out of range, mixed bit-widths or grouping modes, what
 * tmac_mpgemv_fused rejects), TMAC_EHIP. */
enum { TMAC_MULTI_MAX = 8 };
typedef struct {
  const tmac_wdesc* desc;
  const void* packed_dev;
  const void* A_dev;
  int64_t lda;
  const float* act_scale_dev;
  float weight_scale;
  void* out_dev;
  int64_t ldo;
} tmac_gemv_item;
tmac_status tmac_mpgemv_fused_multi(const tmac_gemv_item* items, int32_t count, tmac_act_t act, int32_t N,
                                    tmac_out_t out, void* stream, const tmac_tuning* tuning);

/* Host-side check of a packed blob against a desc (the blob header is the first 256 bytes of what
 * tmac_pack_weights wrote; pass the host copy, or those bytes copied back from the device):
 * TMAC_OK when magic, layout, M, K, bits, g, group, the per-tensor zero point and the sizes in the
 * header are those tmac_pack_weights writes for `desc`; TMAC_EINVAL otherwise (or on a null
 * pointer or an invalid desc).  The device entry points cannot make this check themselves: they
 * never read device memory on the host. */
tmac_status tmac_blob_check(const tmac_wdesc* desc, const void* header_host);

/* Largest tmac_lut_bytes / tmac_workspace_bytes / tmac_fused_workspace_bytes over 1..N_max
 * activation rows: the size of a buffer that serves every call with at most N_max rows (the sizes
 * are not monotonic in N).  0 on bad arguments, or when any N in the range is unsupported for the
 * fused workspace. */
size_t tmac_lut_bytes_max(int32_t N_max, int32_t K, int32_t g, int32_t group, tmac_lut_t lut);
size_t tmac_workspace_bytes_max(const tmac_wdesc* desc, int32_t N_max);
size_t tmac_fused_workspace_bytes_max(const tmac_wdesc* desc, int32_t N_max, tmac_act_t act);

/* tmac_mpgemm for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks and
 * results (bit for bit) as tmac_mpgemm, without the workspace: the split-K partial sums of the
 * batched kernel (layout 3, few activation rows) go to a fixed array of
 * TMAC_NOALLOC_MAX_WORKSPACE bytes inside the library, which every GPU the library runs on holds
 * until the process ends.  The call allocates and frees nothing.
 *   - A call whose partial sums need more (tmac_workspace_bytes(desc, N) - 256 bytes) returns
 *     TMAC_ESIZE before anything is enqueued; tmac_last_error_detail() says so.
 *   - The first call on a GPU looks up that GPU's address of the array (hipGetSymbolAddress): make
 *     it outside stream capture.
 *   - All calls on one GPU share the array: calls that overlap in time on one GPU (two streams)
 *     race.  Its contents mean nothing between calls; nothing in it needs to start at zero. */
#define TMAC_NOALLOC_MAX_WORKSPACE (8u << 20)
tmac_status tmac_mpgemm_noalloc(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev,
                                tmac_lut_t lut, int32_t N, const float* act_scale_dev,
                                float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                void* stream);

const char* tmac_status_str(tmac_status s);

/* Text of the last HIP error this thread met inside the library, or of the last refusal that
 * carries an explanation ("" if none); diagnostics for a TMAC_EHIP or TMAC_ESIZE return. */
const char* tmac_last_error_detail(void);

/* Library version: 1000*major + minor. */
int32_t tmac_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TMAC_H_ */
