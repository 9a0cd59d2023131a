// Host-side preparation of a topology: validation of the two-level CSR, the reverse
// link -> (commodity, candidate set) CSR in its two device layouts (pairs for the resident
// kernel, flat octets plus single pairs for the streaming kernels), and the repacking of the
// forward CSR into self-contained records.  No HIP calls here.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/nimble_plan.h"

namespace nimble {

// ---- reverse CSR ------------------------------------------------------------------------
// One 8-byte pair per (link, commodity, window of 32 candidates) that has at least one
// candidate through the link:
//   word A: bits 0..23 commodity, bits 24..25 window (candidates 32w .. 32w+31),
//           bit 31 = first pair of this commodity in this link's row
//   word B: bit j = candidate 32w+j of the commodity uses the link
// Inside a row pairs ascend by (commodity, window); since a commodity routes on exactly one
// candidate per iteration, at most one pair of a commodity hits, so summing the demands of
// the hit pairs in row order is the sequential order of Algorithm 1's L_e += f.
constexpr uint32_t kCommMask = (1u << 24) - 1u;
constexpr int kWindowShift = 24;
constexpr uint32_t kFirstFlag = 1u << 31;
constexpr int32_t kMaxComm = (1 << 24) - 2;   // one id is kept as the padding sentinel
constexpr int32_t kMaxPathsPerComm = 127;     // four windows of 32, index 255 never occurs
constexpr int32_t kRowLanesHost = 16;         // lanes of one DPP row reduce one single-pair chunk
constexpr int32_t kPairAlign = 2;             // rows are padded to 16 bytes (2 pairs)

// Streaming layout of the same rows.  Commodity ids that fall into one aligned-by-4 window of 8
// consecutive ids are packed into an OCTET: one base id and eight masks (0 for commodities
// that do not use the link), so that one 8-byte load fetches all eight choices.  A row is
// packed in three passes: (1) octets over commodity ids that hold at least kOctetMinFill
// pairs; (2) the left-overs (rows whose commodities are far apart in id order, e.g. "all
// sources towards one destination") get a second chance under a second numbering sigma of the
// commodities -- walking the rows in order, every left-over commodity that has no sigma yet
// receives the next one, so the left-overs of the first row that lists them become
// consecutive and rows with the same left-overs are dense under sigma; octets over sigma read
// a second copy of the choices (and demands) stored in sigma order; (3) what is still left
// becomes octets over ids of any fill.  Only commodities with more than 32 candidates
// (several windows) stay SINGLE pairs.
//
// All octets of all rows form one flat array, row after row, processed 64 at a time (one per
// lane, a "pass").  The low bits of the base word carry two flags: bit 0 = this octet starts a
// new partial-sum slot (first octet of a row, or of a pass), bit 1 = numbered by sigma.  The
// slots of a row are consecutive; pass_first_slot gives the slot of the first octet of a pass.
// Padding octets (no masks, no flags) extend the last slot of their pass by +0.0.
constexpr int32_t kOctetMinFill = 3;
constexpr uint32_t kOctNewSlot = 1u;
constexpr uint32_t kOctSigma = 2u;
constexpr int32_t kSinglesPerLane = 8;        // a single-pair chunk holds 16 * 8 pairs

// Tiles.  Where a row holds many commodities of one WINDOW (kTileIds consecutive ids, or
// consecutive sigma numbers), those commodities are stored as a dense piece of 64 columns x 8
// masks instead of octets: column c covers the commodities window*kTileIds + 8c .. + 7.  One
// work item holds up to kTileRows pieces of the same window (different links); a wave loads
// the 512 choices and demands of the window once, coalesced, and uses them for every row of
// the item, so no per-hit gather is left.  Every piece adds one partial-sum slot to its link.
// A piece whose non-zero masks are all one value is UNIFORM and shrinks to that value plus
// one presence bit per commodity; an item holds pieces of one kind.
// Item descriptor, kTileDescInts int32:
//   [0] first number of the window   [1] bit 0: sigma numbers, bit 1: uniform pieces
//   [2] number of pieces             [3] dense: index of the first piece in tile_mask (2 KiB
//                                        each, lane-contiguous like the masks of a pass);
//                                        uniform: index of the item's block in tile_pres
//   [8..15] slot of piece 0..7 (-1: none)      [16..23] uniform: mask of piece 0..7
// The pieces of a uniform item cover the same commodities; tile_pres holds, per uniform item,
// 64 bytes: byte c, bit s = commodity window + 8c + s is present in the item's pieces.
constexpr int32_t kTileIds = 512;
constexpr int32_t kTileRows = 8;
constexpr int32_t kTileDescInts = 32;
constexpr int32_t kTileMinItems = 128;        // fewest commodities of a window that make a piece
constexpr int64_t kTileAutoPairs = 4000000;   // tiles are used by default from this many pairs on

// Strips.  Short rows that several links share octet for octet (the same commodities, e.g. the
// rail links between two nodes), each with one mask value, leave the octet stream too.  A unit
// is 8 columns (octets) x up to 8 such rows; 8 units fill the 64 lanes of a strip item.  Per
// lane: strip_base (the octet's base word: id | sigma flag), strip_pres (byte r = presence bits
// of the column's 8 commodities in row r of the lane's unit); per unit and row (index
// 8 * unit + row): strip_mask (the row's mask value) and strip_slot (-1: no such row).
constexpr int32_t kStripMinCols = 2;
constexpr int32_t kStripMaxCols = 64;
constexpr int32_t kStripMinRows = 3;

// Link blocks and the order of the rows.  The rows are dealt to blocks of equal weight
// (largest row first, each to the lightest block so far); the flat octet array holds the rows
// block after block, inside a block by ascending link id.  pos_link[i] is the link whose row
// comes i-th, pos_slot_ptr[i] .. pos_slot_ptr[i+1] are its slots.  Every block starts at a pass
// boundary (the tail of its last pass is filled with padding octets that have no masks and
// open no slot), so that one workgroup can reduce the rows of a block into LDS and apply the
// length update of those links right away.  A block holds at most kBlkMaxSlots partial-sum
// slots and kBlkMaxLinks links; a topology that breaks either bound, one with single
// pairs, or one that uses tiles, has no blocks (n_blocks = 0) and runs the separate reduce and update kernels over the
// same arrays.
constexpr int32_t kBlkMaxSlots = 1024;
constexpr int32_t kBlkMaxLinks = 512;

// Link groups (tiled layouts).  The links are cut into groups whose tile items, strip units and
// octets hold rows of the group's links only, and the groups are dealt to blocks of about equal
// work; the rows, items, strips and passes of a block are contiguous in their arrays, and so
// are its partial-sum slots (octet slots; piece and strip slots).  One workgroup can then
// reduce everything its links receive into LDS and apply their length update.  A layout whose
// largest block needs more than kGblkMaxSlots slots has no such blocks (n_gblocks = 0); the
// arrays are the same either way, so the separate reduce and update kernels run on them too.
constexpr int32_t kGblkDescInts = 16;
constexpr int32_t kGblkMaxSlots = 4096;

// ---- forward CSR records ------------------------------------------------------------------
// The forward CSR is repacked into self-contained records of kRecBytes bytes, each holding a
// run of consecutive commodities: a wave fetches one record with four 16-byte loads per lane
// (no pointer chasing), finds in it the global ids of the record's distinct links (whose
// prices it gathers into LDS), the first candidate of every commodity, and for every candidate
// exactly `stride` 8-bit indices into the record's link table.  Paths shorter than the stride
// are padded with the index n_links, whose price slot holds +0.0 (neutral for sum and for max
// of positive prices); the candidates that pad a commodity to a multiple of 4 start with the
// index n_links + 1, whose price slot holds +inf, so their cost is +inf.  The link table comes
// first and always fills kRecTable bytes, stored the way the wave gathers it: 16-byte load l
// holds the links 0*64+l, 1*64+l, 2*64+l, 3*64+l of the table (ascending link ids), entries
// past n_links repeating the last link, so every entry is a valid link id and the gathers need
// nothing but the table.  The body follows; its offsets count from kRecTable:
//   0   int32 k0        first commodity
//   4   int32 p0        first candidate path (global id)
//   8   uint16 nk, np, n_links, off_cp, off_loc, off_sig, off_cq, npad
//   off_sig  int32 sigma[nk]      second numbering of the commodity (-1: none)
//   off_cp   uint16 cp16[nk+1]    first candidate of commodity i, relative to p0
//   off_cq   uint16 cq16[nk+1]    the same with every commodity padded to a multiple of 4
//   off_loc  uint8  loc8[stride][npad]  (index i of every padded candidate, then index i+1,
//                                        ...): four consecutive candidates are one 32-bit word
// Lane-major body (paths of at most kRecLaneSteps links, at least two lanes per commodity): the
// record kernel gives commodity slot g the lanes g*L .. g*L + L - 1 and lane j of a slot the
// candidates 4j .. 4j+3 (quad A) and 4(j+L) .. 4(j+L)+3 (quad B).  The body is then stored so
// that the three 16-byte loads of a lane return exactly that lane's 12 words -- the lane keeps
// them in registers and nothing but the prices goes through LDS:
//   word i     (i < 5)   step i of quad A: the table indices of its four candidates, one byte each
//   word 5 + i (i < 5)   step i of quad B
//   word 10              candidates of the commodity (low byte) | its first candidate relative
//                        to p0, shifted left by 8; 0 for an empty slot
//   word 11              lane 0 of a slot: sigma of the commodity; lane 1 of slot 0:
//                        k0 | nk << 24; lane 1 of slot 1: p0; lane 1 of slot 2: bit 0 = the A
//                        quads of all lanes have the two-by-two product shape, bit 1 = the B
//                        quads (see align_product_quad in host_topo.cpp)
// Load `it` of lane l sits at byte kRecTable + 1024*it + 16*l.  Short paths are padded with
// the index kRecZeroSlot and absent candidates start with kRecInfSlot (their price slots hold
// +0.0 and +inf), so a record has at most kRecMaxLinks table entries in use.
// While link ids fit 16 bits a lane-major record stores its table as 256 uint16 (512 bytes, the
// same gather order: 8-byte load l holds the links l, 64+l, 128+l, 192+l) and is 3.5 KiB long.
// Dictionary format (lane-major bodies, 16-bit tables): words 0..10 of a lane describe how the
// candidates of the record index its link table, not which commodities or links they are, so
// on fabrics built by a product rule (rail x egress x ingress) thousands of records share a few
// dozen bodies.  The bodies then live once in a dictionary (kRecBodyBytes each: load `it` of
// lane l at 1024*it + 16*l as above; word 11, the same in all lanes, says whether the A quads
// (bit 0) and the B quads (bit 1) of the body have the two-by-two product shape, in which the
// record kernel fetches 9 prices per quad instead of 20) that stays in the L2, and a record
// shrinks
// to kRecBytesDict: 16 bytes per lane -- its four 16-bit table entries, its word 11, and the
// number of the record's body (the same in all lanes).  Records are stored sorted by body, so
// a wave that walks a run of records of one body fetches the body once.
constexpr int32_t kRecBytesDict = 1024;
constexpr int32_t kRecBodyBytes = 3 * 1024;
constexpr int32_t kRecTable16 = 512;
constexpr int32_t kRecBytes16 = kRecTable16 + 3 * 1024;
constexpr int32_t kRecLaneWords = 12;
constexpr int32_t kRecLaneSteps = 5;
constexpr int32_t kRecZeroSlot = 254;
constexpr int32_t kRecInfSlot = 255;

#ifndef NIMBLE_REC_KB
#define NIMBLE_REC_KB 4
#endif
constexpr int32_t kRecBytes = 1024 * NIMBLE_REC_KB;   // one 16-byte load per lane and KiB
constexpr int32_t kRecTable = 1024;       // bytes of the link table: 4 gathers x 64 lanes
constexpr int32_t kRecHeader = 24;
constexpr int32_t kRecPriceSlots = 256;   // price slots a wave keeps per record
constexpr int32_t kRecMaxLinks = 254;     // link table entries (8-bit indices); slots n_links and
                                          // n_links + 1 hold +0.0 and +inf
constexpr int32_t kRecMaxStride = 8;      // longest path a record can hold
constexpr int32_t kRecMaxComm = 64;

struct HostTopo {
    int32_t E = 0, K = 0, P = 0;
    int64_t nnz = 0;
    int32_t pmax = 0;       // most candidates of any commodity
    int32_t lmax = 0;       // most links of any path
    std::vector<double> invcap;          // [E] by link id
    std::vector<double> invcap_pos;      // [E] by position (pos_link)
    // reverse CSR in pair units, rows padded to kPairAlign pairs with (commodity K, mask 0)
    std::vector<int32_t> rev_ptr;        // [E+1], padded offsets in pairs
    std::vector<uint32_t> rev_pair;      // [2 * rev_ptr[E]], words A,B interleaved
    std::vector<int32_t> rev_rowlen;     // [E], unpadded row lengths in pairs
    int64_t n_pairs = 0;                 // unpadded total
    // streaming layout
    std::vector<uint32_t> oct_base;      // [n_oct_padded]: base id | flags, padded to 64
    std::vector<uint32_t> oct_mask;      // [8 * n_oct_padded]; per pass: words 0..3 of its 64
                                         // octets lane after lane, then words 4..7
    int64_t n_octets = 0;                // unpadded
    int64_t n_octets_sigma = 0;          // of which numbered by sigma
    std::vector<int32_t> pass_first_slot; // [n_oct_padded / 64]
    int32_t tiles = -1;                  // option: 1 = build tiles, 0 = never, -1 = by size
    int32_t tile_min_items = 0;          // option: fewest commodities per piece (0 = default)
    int32_t n_pieces = 0, n_tile_items = 0;
    int64_t n_piece_items = 0;           // (link, commodity) pairs stored in pieces
    int32_t n_pieces_uniform = 0;
    bool tiles_dense_only = false;       // option: never store a piece as uniform
    std::vector<int32_t> tile_desc;      // [kTileDescInts * n_tile_items]
    std::vector<uint32_t> tile_mask;     // [512 * (dense pieces + 1)]
    std::vector<uint8_t> tile_pres;      // [64 * (uniform items + 1)]
    int32_t n_strip_items = 0, n_strip_rows = 0;
    std::vector<uint32_t> strip_base;    // [64 * (n_strip_items + 1)]
    std::vector<uint64_t> strip_pres;    // [64 * (n_strip_items + 1)]
    std::vector<uint32_t> strip_mask;    // [64 * (n_strip_items + 1)]
    std::vector<int32_t> strip_slot;     // [64 * (n_strip_items + 1)]
    int32_t blk_passes = 0;              // option: target passes per link block (0 = default)
    int32_t n_blocks = 0;                // 0: the topology does not fit link blocks
    std::vector<int32_t> pos_link;       // [E] link of every position of the flat order
    std::vector<int32_t> pos_slot_ptr;   // [E+1] octet slots of a position
    std::vector<int32_t> pos_xslot;      // [2 * E] first and end of the link's other slots
                                         // (pieces, strip units, single-pair chunks), by
                                         // position
    std::vector<int32_t> blk_pos_ptr;    // [n_blocks+1] first position of a block
    std::vector<int32_t> blk_pass_ptr;   // [n_blocks+1] first pass of a block
    std::vector<int32_t> blk_desc;       // [8 * n_blocks] what one workgroup of the fused kernel
                                         // needs: first and end position, first and end pass,
                                         // first slot, three zeros
    int32_t link_groups = -1;            // option: 0 = no link groups, else build them where
                                         // the layout is tiled
    int32_t grp_target = 0;              // option: blocks to deal the groups to (0: 256)
    int32_t n_gblocks = 0;               // blocks of link groups (0: none)
    std::vector<int32_t> gblk_desc;      // [kGblkDescInts * n_gblocks], see host_topo.cpp
    int32_t gblk_max_slots = 0;          // most partial-sum slots of a block
    int32_t gblk_max_tasks = 0;          // most tile items + strip items + passes of a block
    int32_t n_oct_slots = 0;
    std::vector<int32_t> sigma;          // [K] second numbering, -1 = none
    int32_t sigma_size = 0;              // length of the sigma-ordered copies (multiple of 8)
    std::vector<uint32_t> single_pair;   // [2 * n_singles_padded], rows padded to 2 pairs
    int64_t n_single_pairs = 0;          // unpadded
    std::vector<int32_t> schunk_begin, schunk_end, schunk_slot;   // pair units
    int32_t n_slots = 0;                 // octet slots + single-chunk slots
    // forward records (n_records = 0 when the topology does not fit them: a path longer than
    // kRecMaxStride links, padding above 1.5x, or a commodity that alone overflows a record)
    int32_t rec_comm_cap = 0;            // option: most commodities per record (0: one round of
                                         // the record kernel, 64 / rec_lanes)
    int32_t rec_lanes = 0;               // lanes per commodity the record kernel should use
    int32_t rec_stride = 0;              // indices per candidate = lmax
    int32_t rec_lane_major = 1;          // option in, layout out: the body of a record is laid
                                         // out lane by lane (see kRecLaneWords)
    int32_t rec_table16 = 1;             // option in, layout out: 16-bit link tables
    int32_t rec_dict = -1;               // option in (-1: when it pays, 0: never, 1: whenever
                                         // the format allows), layout out (0 / 1): bodies in a
                                         // dictionary, records of kRecBytesDict
    int32_t rec_product_quads = 1;       // option: 0 = never store quads in the two-by-two
                                         // product shape (see align_product_quad)
    int32_t n_bodies = 0;                // distinct bodies
    int32_t n_bodies_product = 0;        // of which with all quads in the product shape
    int64_t rec_price_reads = 0;         // lane-major records: price reads per lane, summed
                                         // over the records (9 or 4 * stride per quad)
    std::vector<uint32_t> rec_dict_words; // [n_bodies * kRecBodyBytes / 4]
    std::vector<int32_t> rec_body;       // [n_records] body of every record (ascending)
    int32_t rec_bytes = 0;               // bytes of a record: kRecBytes, kRecBytes16 or
                                         // kRecBytesDict
    int32_t n_records = 0;
    int32_t rec_max_links = 0;           // largest link table of any record
    std::vector<uint8_t> records;        // [n_records * kRecBytes]
};

// Checks every documented precondition.  Returns NIMBLE_OK or the error; `why` gets the text.
nimble_status_t validate_csr(int32_t n_links, const double *cap, int32_t n_comm,
                             const int32_t *comm_path_ptr, int32_t n_paths,
                             const int32_t *path_link_ptr, const int32_t *path_links,
                             std::string &why);

// Reads the layout options of `out` from the NIMBLE_TUNE_* environment variables (record
// capacity, link block size, tiles on/off, piece threshold); unset variables leave defaults.
void read_layout_options(HostTopo &out);

// Builds everything in HostTopo from validated input.  out.rec_comm_cap,
// out.blk_passes, out.tiles and out.tile_min_items are read as options.
void build_host_topo(int32_t n_links, const double *cap, int32_t n_comm,
                     const int32_t *comm_path_ptr, int32_t n_paths,
                     const int32_t *path_link_ptr, const int32_t *path_links,
                     HostTopo &out);

// The forward records alone (build_host_topo calls it last): needs out.pmax, out.lmax, out.nnz
// and out.sigma.
void build_forward_records(int32_t n_links, int32_t n_comm, const int32_t *comm_path_ptr,
                           int32_t n_paths, const int32_t *path_link_ptr,
                           const int32_t *path_links, HostTopo &out);

}  // namespace nimble
