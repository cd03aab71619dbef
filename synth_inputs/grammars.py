"""Grammar texts used by the synthetic workloads.

Dialect (a small EBNF): ``name ::= alternatives``; alternatives separated by
``|``; items are ``"literal"`` (escapes ``\\" \\\\ \\n \\t \\r \\xHH \\uHHHH``),
character classes ``[a-z0-9_]`` / negated ``[^...]`` over Unicode code points
(same escapes plus ``\\] \\- \\^``), rule names, groups ``( ... )`` and the
postfix operators ``* + ?``; ``#`` starts a comment.  A rule ends where the
next ``name ::=`` begins.

Everything here is text (or a plain dict describing a schema); nothing is
parsed or interpreted in this module.
"""

from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------
# Workload 1: arithmetic, 5 rules.  Spaces may separate lexemes but never sit
# inside a digit run, and never lead or trail the whole expression.
# ---------------------------------------------------------------------------
ARITH_GRAMMAR = r"""
expr   ::= term (ws "+" ws term)*
term   ::= factor (ws "*" ws factor)*
factor ::= digit+ | "(" ws expr ws ")"
digit  ::= [0-9]
ws     ::= " "*
"""

# ---------------------------------------------------------------------------
# Workload 2: generic JSON (ECMA-404 shape).
# ---------------------------------------------------------------------------
JSON_GRAMMAR = r"""
root    ::= ws value ws
value   ::= object | array | string | number | "true" | "false" | "null"
object  ::= "{" ws ( member ( ws "," ws member )* ws )? "}"
member  ::= string ws ":" ws value
array   ::= "[" ws ( value ( ws "," ws value )* ws )? "]"
string  ::= "\"" char* "\""
char    ::= [^"\\\x00-\x1f] | "\\" escape
escape  ::= ["\\/bfnrt] | "u" hex hex hex hex
hex     ::= [0-9a-fA-F]
number  ::= "-"? int frac? exp?
int     ::= "0" | [1-9] [0-9]*
frac    ::= "." [0-9]+
exp     ::= [eE] [+\-]? [0-9]+
ws      ::= [ \t\n\r]*
"""

# ---------------------------------------------------------------------------
# A markup grammar in the style of XML (context-free: closing names are not
# matched against opening names).  Elements, attributes with two quote styles,
# text, entity references, comments, self-closing tags.
# ---------------------------------------------------------------------------
XML_GRAMMAR = r"""
root     ::= ws element ws
element  ::= "<" name attrs ws ( "/>" | ">" content "</" name ws ">" )
attrs    ::= ( ws1 name ws "=" ws value )*
value    ::= "\"" [^"<&]* "\"" | "'" [^'<&]* "'"
content  ::= ( element | text | entity | comment )*
text     ::= [^<&]+
entity   ::= "&" name ";" | "&#" [0-9]+ ";"
comment  ::= "<!--" ( [^\-] | "-" [^\-] )* "-->"
name     ::= [A-Za-z_] [A-Za-z0-9_.\-]*
ws       ::= [ \t\n]*
ws1      ::= [ \t\n]+
"""

# ---------------------------------------------------------------------------
# A small scripting language in the style of Python, kept context-free by
# giving every compound statement a one-line body.  Every sentence is also a
# Python module (names start with one of x z u v or an underscore, so none
# is a keyword; integers have no leading zeros; attribute access never follows
# a number).  Word operators ("not in", "is not", "if ... else") next to
# names and the two quote styles give the walks alternatives to carry.
# ---------------------------------------------------------------------------
PYDSL_GRAMMAR = r"""
root     ::= line (nl line)* nl?
nl       ::= "\n"+
line     ::= stmt (sp "#" [^\n\x00-\x1f]*)?
stmt     ::= simple | "if " expr ":" sp simple (nl "elif " expr ":" sp simple)* (nl "else:" sp simple)?
           | "while " expr ":" sp simple | "for " name " in " expr ":" sp simple
           | "def " name "(" sp (name (sp "," sp name)*)? sp "):" sp simple
simple   ::= small (sp ";" sp small)*
small    ::= "pass" | "break" | "continue" | "return" (" " expr)? | target sp assignop sp expr | expr
target   ::= name ( "." name | "[" sp expr sp "]" )*
assignop ::= "=" | "+=" | "-=" | "*=" | "/=" | "//=" | "%="
expr     ::= "lambda" (" " name (sp "," sp name)*)? ":" sp expr | ternary
ternary  ::= or_e (" if " or_e " else " expr)?
or_e     ::= and_e (" or " and_e)*
and_e    ::= not_e (" and " not_e)*
not_e    ::= "not " not_e | cmp
cmp      ::= arith (cmpop arith)*
cmpop    ::= sp ("==" | "!=" | "<=" | ">=" | "<" | ">") sp | " in " | " not in " | " is " | " is not "
arith    ::= term (sp [+\-] sp term)*
term     ::= factor (sp ("*" | "//" | "/" | "%") sp factor)*
factor   ::= [+\-~] factor | power
power    ::= atom (sp "**" sp factor)?
atom     ::= primary trailer* | number | string | "True" | "False" | "None"
primary  ::= name | "(" sp expr sp ")" | "[" sp (expr (sp "," sp expr)*)? sp "]"
           | "{" sp (expr sp ":" sp expr (sp "," sp expr sp ":" sp expr)*)? sp "}"
trailer  ::= "(" sp (expr (sp "," sp expr)*)? sp ")" | "[" sp expr sp "]" | "." name
name     ::= [xzuv_] [A-Za-z0-9_]*
number   ::= ("0" | [1-9] [0-9]*) ("." [0-9]+)?
string   ::= "\"" ([^"\\\n\x00-\x1f] | "\\" ["\\'nt])* "\"" | "'" ([^'\\\n\x00-\x1f] | "\\" ["\\'nt])* "'"
sp       ::= " "*
"""

# ---------------------------------------------------------------------------
# Workload 4(ii): a C/SQL-like language, about 60 rules.  Iterative (never
# left-recursive) precedence chain, keywords, identifiers, literals with
# escapes, blocks and embedded SELECT statements.
# ---------------------------------------------------------------------------
CSQL_GRAMMAR = r"""
root         ::= ws (item ws)*
item         ::= func_def | decl_stmt | struct_def | query_stmt
func_def     ::= type sp ident ws "(" ws params? ws ")" ws block
params       ::= param (ws "," ws param)*
param        ::= type sp ident
struct_def   ::= "struct" sp ident ws "{" ws (field ws)* "}" ws ";"
field        ::= type sp ident ws ";"
type         ::= base_type (ws "*")*
base_type    ::= "int" | "char" | "float" | "double" | "void" | "long" | "short" | "bool" | "unsigned" sp "int" | "struct" sp ident
block        ::= "{" ws (stmt ws)* "}"
stmt         ::= block | if_stmt | while_stmt | do_stmt | for_stmt | switch_stmt | return_stmt | break_stmt | continue_stmt | goto_stmt | decl_stmt | expr_stmt | query_stmt
if_stmt      ::= "if" ws "(" ws expr ws ")" ws stmt (ws "else" ws stmt)?
while_stmt   ::= "while" ws "(" ws expr ws ")" ws stmt
do_stmt      ::= "do" ws block ws "while" ws "(" ws expr ws ")" ws ";"
for_stmt     ::= "for" ws "(" ws expr? ws ";" ws expr? ws ";" ws expr? ws ")" ws stmt
switch_stmt  ::= "switch" ws "(" ws expr ws ")" ws "{" ws (case_clause ws)* "}"
case_clause  ::= ("case" sp expr | "default") ws ":" ws (stmt ws)*
return_stmt  ::= "return" (sp expr)? ws ";"
break_stmt   ::= "break" ws ";"
continue_stmt ::= "continue" ws ";"
goto_stmt    ::= "goto" sp ident ws ";"
decl_stmt    ::= type sp declarator (ws "," ws declarator)* ws ";"
declarator   ::= ident (ws "[" ws int_lit? ws "]")* (ws "=" ws assign)?
expr_stmt    ::= expr ws ";"
expr         ::= assign (ws "," ws assign)*
assign       ::= ternary (ws assign_op ws assign)?
assign_op    ::= "=" | "+=" | "-=" | "*=" | "/=" | "%=" | "&=" | "|=" | "^=" | "<<=" | ">>="
ternary      ::= lor (ws "?" ws expr ws ":" ws ternary)?
lor          ::= land (ws "||" ws land)*
land         ::= bor (ws "&&" ws bor)*
bor          ::= bxor (ws "|" ws bxor)*
bxor         ::= band (ws "^" ws band)*
band         ::= equality (ws "&" ws equality)*
equality     ::= relational (ws ("==" | "!=") ws relational)*
relational   ::= shift (ws ("<=" | ">=" | "<" | ">") ws shift)*
shift        ::= additive (ws ("<<" | ">>") ws additive)*
additive     ::= mult (ws [+\-] ws mult)*
mult         ::= unary (ws [*/%] ws unary)*
unary        ::= unary_op ws unary | "sizeof" ws "(" ws type ws ")" | postfix
unary_op     ::= "!" | "~" | "-" | "+" | "*" | "&" | "++" | "--"
postfix      ::= primary (ws postfix_op)*
postfix_op   ::= "(" ws args? ws ")" | "[" ws expr ws "]" | "." ws ident | "->" ws ident | "++" | "--"
args         ::= assign (ws "," ws assign)*
primary      ::= ident | float_lit | int_lit | string_lit | char_lit | "(" ws expr ws ")" | "NULL" | "true" | "false"
ident        ::= [A-Za-z_] [A-Za-z0-9_]*
int_lit      ::= "0" [xX] [0-9a-fA-F]+ | [0-9]+ [uUlL]?
float_lit    ::= [0-9]+ "." [0-9]* float_exp? [fF]? | "." [0-9]+ float_exp? [fF]? | [0-9]+ float_exp [fF]?
float_exp    ::= [eE] [+\-]? [0-9]+
string_lit   ::= "\"" str_char* "\""
str_char     ::= [^"\\\n] | "\\" esc
char_lit     ::= "'" ([^'\\\n] | "\\" esc) "'"
esc          ::= [nrt0\\'"abfv] | "x" [0-9a-fA-F] [0-9a-fA-F]
query_stmt   ::= query ws ";"
query        ::= select_q | insert_q | update_q | delete_q
select_q     ::= "SELECT" sp ("DISTINCT" sp)? select_list sp "FROM" sp table_list (sp join_clause)* (sp where_clause)? (sp group_clause)? (sp order_clause)? (sp limit_clause)?
select_list  ::= "*" | select_item (ws "," ws select_item)*
select_item  ::= sql_expr (sp "AS" sp ident)?
table_list   ::= table_ref (ws "," ws table_ref)*
table_ref    ::= ident (sp "AS" sp ident)?
join_clause  ::= (("LEFT" | "RIGHT" | "INNER") sp)? "JOIN" sp table_ref sp "ON" sp sql_expr
where_clause ::= "WHERE" sp sql_expr
group_clause ::= "GROUP" sp "BY" sp column (ws "," ws column)* (sp "HAVING" sp sql_expr)?
order_clause ::= "ORDER" sp "BY" sp order_item (ws "," ws order_item)*
order_item   ::= column (sp ("ASC" | "DESC"))?
limit_clause ::= "LIMIT" sp [0-9]+ (sp "OFFSET" sp [0-9]+)?
insert_q     ::= "INSERT" sp "INTO" sp ident ws "(" ws column (ws "," ws column)* ws ")" ws "VALUES" ws "(" ws sql_expr (ws "," ws sql_expr)* ws ")"
update_q     ::= "UPDATE" sp ident sp "SET" sp set_item (ws "," ws set_item)* (sp where_clause)?
set_item     ::= column ws "=" ws sql_expr
delete_q     ::= "DELETE" sp "FROM" sp ident (sp where_clause)?
sql_expr     ::= sql_and (sp "OR" sp sql_and)*
sql_and      ::= sql_not (sp "AND" sp sql_not)*
sql_not      ::= ("NOT" sp)? sql_cmp
sql_cmp      ::= sql_term (ws ("<>" | "<=" | ">=" | "=" | "<" | ">") ws sql_term | sp "LIKE" sp sql_string | sp "IS" sp ("NOT" sp)? "NULL" | sp "IN" ws "(" ws sql_term (ws "," ws sql_term)* ws ")")?
sql_term     ::= sql_atom (ws [+\-*/] ws sql_atom)*
sql_atom     ::= column | [0-9]+ ("." [0-9]+)? | sql_string | ident ws "(" ws ("*" | sql_expr (ws "," ws sql_expr)*)? ws ")" | "(" ws sql_expr ws ")"
column       ::= ident ("." ident)?
sql_string   ::= "'" ([^'] | "''")* "'"
sp           ::= [ \t\n]+
ws           ::= [ \t\n]*
"""

# ---------------------------------------------------------------------------
# Workloads 3 and 5: grammar text derived from a seeded random schema.
# ---------------------------------------------------------------------------
_SHARED_SCHEMA_RULES = r"""
string  ::= "\"" chars "\""
chars   ::= char*
char    ::= [^"\\\x00-\x1f] | "\\" escape
escape  ::= ["\\/bfnrt] | "u" hex hex hex hex
hex     ::= [0-9a-fA-F]
integer ::= "-"? int
number  ::= "-"? int frac? exp?
int     ::= "0" | [1-9] [0-9]*
frac    ::= "." [0-9]+
exp     ::= [eE] [+\-]? [0-9]+
boolean ::= "true" | "false"
ws      ::= [ \t\n\r]*
"""

_KEY_ALPHABET = "abcdefghijklmnopqrstuvwxyz_"


def _rand_name(rng: np.random.Generator, lo: int, hi: int) -> str:
    n = int(rng.integers(lo, hi + 1))
    return "".join(_KEY_ALPHABET[int(j)] for j in rng.integers(0, len(_KEY_ALPHABET), size=n))


def random_schema(seed: int, max_depth: int = 4, string_heavy: bool = False) -> dict:
    """A seeded random schema as a plain nested dict.

    Objects have 8-20 properties with distinct random keys ``[a-z_]{3,12}``
    in a fixed order; property types are string / integer / number / boolean
    / enum (3-8 string values) / array / object (only above ``max_depth``).
    With ``string_heavy`` at least 60 % of the leaves are strings or enums.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if string_heavy:
        leaf_types = ["string", "enum", "integer", "number", "boolean"]
        leaf_p = [0.50, 0.22, 0.10, 0.08, 0.10]
    else:
        leaf_types = ["string", "enum", "integer", "number", "boolean"]
        leaf_p = [0.30, 0.15, 0.20, 0.15, 0.20]

    def leaf() -> dict:
        t = leaf_types[int(rng.choice(len(leaf_types), p=leaf_p))]
        if t == "enum":
            k = int(rng.integers(3, 9))
            vals = []
            while len(vals) < k:
                v = _rand_name(rng, 2, 10)
                if v not in vals:
                    vals.append(v)
            return {"type": "enum", "values": vals}
        return {"type": t}

    def value(depth: int) -> dict:
        u = rng.random()
        if depth < max_depth and u < 0.10:
            return obj(depth + 1)
        if u < 0.22:
            item = obj(depth + 1) if (depth < max_depth and rng.random() < 0.15) else leaf()
            return {"type": "array", "items": item}
        return leaf()

    def obj(depth: int) -> dict:
        k = int(rng.integers(8, 21))
        keys = []
        while len(keys) < k:
            name = _rand_name(rng, 3, 12)
            if name not in keys:
                keys.append(name)
        return {"type": "object", "properties": [(name, value(depth)) for name in keys]}

    return obj(1)


def make_schema_grammar(seed: int, max_depth: int = 4, string_heavy: bool = False) -> str:
    """Grammar text for ``random_schema(seed, ...)``; root rule is ``root``."""
    schema = random_schema(seed, max_depth=max_depth, string_heavy=string_heavy)
    rules = []
    counter = [0]

    def fresh(prefix: str) -> str:
        counter[0] += 1
        return f"{prefix}_{counter[0]}"

    def emit(node: dict) -> str:
        t = node["type"]
        if t in ("string", "integer", "number", "boolean"):
            return t
        if t == "enum":
            name = fresh("enum")
            alts = " | ".join('"\\"' + v + '\\""' for v in node["values"])
            rules.append(f"{name} ::= {alts}")
            return name
        if t == "array":
            item = emit(node["items"])
            name = fresh("arr")
            rules.append(f'{name} ::= "[" ws ( {item} ( ws "," ws {item} )* ws )? "]"')
            return name
        if t == "object":
            name = fresh("obj")
            parts = []
            for i, (key, sub) in enumerate(node["properties"]):
                ref = emit(sub)
                sep = 'ws "," ws ' if i else ""
                parts.append(f'{sep}"\\"{key}\\"" ws ":" ws {ref}')
            rules.append(f'{name} ::= "{{" ws ' + " ".join(parts) + ' ws "}"')
            return name
        raise ValueError(t)

    top = emit(schema)
    text = f"root ::= ws {top} ws\n" + "\n".join(rules) + "\n" + _SHARED_SCHEMA_RULES
    return text
