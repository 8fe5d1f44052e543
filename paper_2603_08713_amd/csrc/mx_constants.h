// Sizes the whole library agrees on (plain C++, no device code).
#pragma once

namespace mx {

constexpr int kBlock = 32;   // elements per E8M0 scale (Sec. 2.2)
constexpr int kMacro = 128;  // elements per MBS word (Sec. 4.3)
constexpr int kWave = 64;

}  // namespace mx
