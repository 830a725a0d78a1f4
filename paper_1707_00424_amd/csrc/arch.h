// Host-side description of the networks: resolved sizes and the packing of one replica row.
#pragma once
#include <string>
#include <vector>

#include "common.h"

struct Arch {
  int model = 0;
  int H = 0, W = 0, C = 0, classes = 0;
  int a0 = 0, a1 = 0, a2 = 0, a3 = 0;  // model-specific sizes after defaults
  int bn = 0;                          // LeNet: batch-norm after conv1, conv2 and fc1
};

struct Segment {
  std::string name;
  int64_t offset = 0, size = 0;
  int kind = 0;
  int shape[4] = {0, 0, 0, 0};
  int fan_in = 0;
};

struct WrnBlock {
  std::string name;
  int cin, cout, stride;
  bool has_sc;
};

// Fills defaults and validates; returns false (with msg) on a bad configuration.
bool resolve_arch(const parle_config &cfg, Arch &a, std::string &msg);
// Segments of one replica row in execution order, weight before bias.
std::vector<Segment> build_layout(const Arch &a);
std::vector<WrnBlock> wrn_block_list(const Arch &a);
// Index of the segment called `name`, or -1.
int find_segment(const std::vector<Segment> &segs, const std::string &name);
