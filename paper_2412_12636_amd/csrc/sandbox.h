// Internal view of the record / replay hook for the stage sequencing code.
#pragma once
struct tm_comm;
namespace tmk {
// true when calls of this scope are stored or served from the tape (the stage then keeps the tensor separate)
bool comm_intercepts(const tm_comm *c, int scope);
}  // namespace tmk
