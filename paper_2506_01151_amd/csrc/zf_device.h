// Plain-data layouts shared by the host code and the HIP kernels.
#pragma once
#include <stdint.h>

namespace zf {

// Encoding of the symbol that follows the dot at a dotted position.
enum : uint16_t {
    SYM_KIND_SHIFT = 14,
    SYM_NT = 0,        // low 13 bits: nonterminal id; bit 13: the nonterminal is nullable
    SYM_TERM = 1,      // low 14 bits: terminal id
    SYM_END = 2,       // dot at the end of the rule; low 14 bits: lhs nonterminal
    SYM_NULLABLE_BIT = 1u << 13,
    SYM_ID_MASK_NT = (1u << 13) - 1,
    SYM_ID_MASK = (1u << 14) - 1,
    DFA_DEAD = 0xFFFF,
};
// Item word used on the device: bits 0-13 dotted position, bit 14 = completed ("lhs complete since
// origin"), bit 15 = the postdot symbol is a terminal and bits 16-31 hold its DFA state; for an item
// that waits for a nonterminal Y: bit 16 = Y is nullable, bits 17-29 = Y.
enum : uint32_t {
    IW_POS_MASK = 0x3FFF, IW_END = 0x4000, IW_TERM = 0x8000,
    IW_NT_NULLABLE = 1u << 16, IW_NT_SHIFT = 17, IW_NT_MASK = 0x1FFF,
    MAX_POSITIONS = 0x3FFF,
    COMP_ADVANCE_WAITING = 0xFFFF,   // entry of the completion lists (host form)
};
// Per-DFA-state word.  States of a literal terminal form a chain (one expected byte, next state
// q + 1) and need no table row: flags | QF_LITERAL | expected byte << 8 | flags of state q+1 << 16.
// Other states: flags | dense transition row << 16; a row entry is next state | its flags << 16.
enum : uint8_t { QF_ACCEPT = 1, QF_CONT = 2, QF_LITERAL = 4 };

// One Earley item.  p: dotted position (index into sym[]); q: DFA state when the postdot
// symbol is a terminal (global state numbering, so q also names the terminal), else 0;
// o: index of the set the rule started in (the classic origin).
struct Item {
    uint16_t p, q;
    uint32_t o;
};

// One trie node, preorder layout.  skip = index of the first node after this subtree.
// rank = number of string-carrying nodes before this one (so a node that carries a string
// owns bit `rank` of the rank-ordered verdict bitmap).
struct TrieNode {
    uint32_t skip;
    uint32_t rank;
    uint8_t byte, depth, has_string, cls;   // cls = byte equivalence class of `byte`
    uint32_t n_sub;      // strings carried by this node's subtree (itself included)
};

struct alignas(16) Str16 { uint32_t w[4]; };       // 16 one-byte symbols, first symbol in the low byte of w[0]

static const int MAX_TOKEN_LEN_ON_DEVICE = 255;   // deeper nodes never occur: depth is a uint8
static const int TOK_LEN_LONG = 255;               // DeviceTables::tok_len of a token longer than the 16 classes tok16 holds
static const int CHUNK_ANC = 16;                  // ancestors stored per chunk (longer paths use parent links)

// Immutable per-engine tables in device memory.  Every array is padded to a multiple of 16 bytes
// so that a block can stage it into LDS with 4-byte copies.
struct DeviceTables {
    const uint32_t *advpq;      // [P] the item word to insert when the dot arrives at position p
    const uint8_t *cls;         // [256] byte -> class
    const uint32_t *qinfo;      // [Q]
    const uint32_t *scan_off;   // [N*n_cls+1] CSR into scan_list
    const uint32_t *comp_off;   // [N*N+1] CSR into comp_list
    const uint32_t *delta;      // [dense rows][n_cls] next state | flags << 16, DFA_DEAD in the low half = no edge
    const uint32_t *scan_list;  // pairs: item word (terminal already stepped once), flags of its DFA state
    const uint32_t *comp_list;  // item words the completion adds; 0xFFFFFFFF: advance the waiting item itself
    const uint8_t *table_blob;  // the eight tables above are one allocation in this order, each padded to 16 bytes
    uint32_t small_bytes[5];    // padded byte sizes of advpq .. comp_off (always staged into LDS when they fit)
    uint32_t big_bytes[3];      // padded byte sizes of delta, scan_list, comp_list
    const TrieNode *nodes;      // [n_nodes]
    const uint32_t *parent;     // [n_nodes] parent node index, 0xFFFFFFFF for depth-1 nodes
    const uint32_t *chunk_begin; // [n_chunks] first node of the chunk
    const uint32_t *chunk_end;   // [n_chunks] one past the last string node of the chunk
    const TrieNode *chunk_anc;   // [n_chunks][CHUNK_ANC] copies of the ancestors of the chunk's first node, depth 1 first
    const uint32_t *rank_of;    // [V] rank of token v's string, 0xFFFFFFFF for the empty token
    // The distinct strings in rank order as strings of byte classes (the mask-automaton kernel reads
    // a string front to back, one lane per string):
    const uint32_t *str_off;    // [n_strings + 1] offsets into str_cls
    const uint8_t *str_cls;     // classes of the strings' bytes, flat
    const Str16 *str16;         // [n_strings] the first 16 classes of each string (zero padded), one aligned load
    const uint8_t *cls_rep;     // [n_cls] one byte of each class (every DFA treats the bytes of a class alike)
    // Context-independent token-mask cache (paper Section 4.3), one bitset row of Wr words per DFA
    // state q (row q) and per nonterminal Y (row Q + Y), in string-rank order:
    const uint32_t *ci_valid;   // strings a terminal entered in state q swallows whole
    const uint32_t *ci_cd;      // strings on which that terminal dies after passing an accepting state
    // The same per TOKEN, for the mask kernel over the persistent automaton, which works in token order and writes the
    // caller's mask rows itself (null unless the engine runs that kernel):
    const Str16 *tok16;         // [V] the first 16 byte classes of token v's string (zero padded)
    const uint8_t *tok_len;     // [V] length of token v's string; 0 = the empty token (never allowed), TOK_LEN_LONG = more than 16 bytes (see rank_of / str_off)
    const uint32_t *ci_valid_tok; // [Q + N][W] the rows of ci_valid with bit v = the verdict on token v's string
    const uint32_t *ci_cd_tok;    // [Q + N][W] likewise for ci_cd
    int32_t Q;
    int32_t N, n_cls, end_base, n_nodes, n_chunks, n_strings, V, W;
    int32_t chunk_ranks;        // strings per chunk: 8, 16 or 32
    int32_t Wr;                 // 32-bit words per row of the rank-ordered verdict bitmap
};

// Per-row header of the uploaded chart.  Items of set k: items[item_base + set_off[set_base+k] ..
// item_base + set_off[set_base+k+1]).
struct RowChart {
    uint32_t n_sets;     // m; the last set (m-1) is the current one
    uint32_t set_base;   // index into the shared set_off array
    uint32_t item_base;  // index into the shared item array
    uint32_t ent_base;   // index into the shared entry array: bitset rows of the current set's items
    uint32_t n_ent;      // 0 = token-mask cache not used for this row
    uint32_t n_items;    // items of the row's chart
    uint32_t pad[2];
};

}  // namespace zf
